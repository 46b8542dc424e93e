// okt_region_partition: balanced split of the index space by the local top-k
// entries (Algorithm 1, lines 5-7; Sec. 3.1.1).
//
// The sorted COO index list is its own cumulative distribution: the r-th of R
// equal-count quantiles is the index stored at position floor(r * nnz / R).
// O(R) gathers and O(R log nnz) probes; latency only.
#include "okt_device.h"

namespace okt {

__device__ __forceinline__ uint64_t lower_bound_u32(const uint32_t* a, uint64_t len, uint32_t x) {
    uint64_t lo = 0, hi = len;
    while (lo < hi) {
        const uint64_t mid = lo + ((hi - lo) >> 1);
        if (a[mid] < x) lo = mid + 1; else hi = mid;
    }
    return lo;
}

__global__ __launch_bounds__(256) void partition_kernel(
    const uint32_t* __restrict__ idx, const uint64_t* __restrict__ d_nnz, uint64_t n, uint32_t R,
    uint32_t* __restrict__ bounds, uint64_t* __restrict__ offsets) {
    const uint64_t nnz = *d_nnz;
    for (uint64_t r = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; r <= R;
         r += (uint64_t)gridDim.x * blockDim.x) {
        uint32_t b;
        uint64_t off;
        if (r == 0) {
            b = 0; off = 0;
        } else if (r == R) {
            b = (uint32_t)n; off = nnz;
        } else if (nnz == 0) {
            b = (uint32_t)((r * n) / R); off = 0;      // the naive equal split
        } else {
            b = idx[(r * nnz) / R];                    // r, nnz < 2^32: no overflow
            off = lower_bound_u32(idx, nnz, b);
        }
        bounds[r] = b;
        offsets[r] = off;
    }
}

}  // namespace okt

extern "C" int okt_region_partition(const uint32_t* d_idx, const uint64_t* d_nnz, uint64_t n,
                                    uint32_t R, uint32_t* d_bounds_out, uint64_t* d_offsets_out,
                                    void* stream) {
    using namespace okt;
    if (!d_idx || !d_nnz || !d_bounds_out || !d_offsets_out) return OKT_ERR_INVALID_ARG;
    if (n == 0 || n > 0xffffffffull || R == 0) return OKT_ERR_INVALID_ARG;
    if (!aligned(d_nnz, 8) || !aligned(d_offsets_out, 8) || !aligned(d_idx, 4) ||
        !aligned(d_bounds_out, 4)) return OKT_ERR_INVALID_ARG;
    uint64_t blocks = ((uint64_t)R + 1 + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    timing_before((hipStream_t)stream);
    hipLaunchKernelGGL(partition_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       (hipStream_t)stream, d_idx, d_nnz, n, R, d_bounds_out, d_offsets_out);
    timing_after((hipStream_t)stream);
    return launch_status();
}
