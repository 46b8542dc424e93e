// okt_region_partition: balanced split of the index space by the local top-k
// entries (Algorithm 1, lines 5-7; Sec. 3.1.1).
//
// The sorted COO index list is its own cumulative distribution: the r-th of R
// equal-count quantiles is the index stored at position floor(r * nnz / R).
// O(R) gathers and O(R log nnz) probes; latency only.
#include "okt_device.h"
#include "okt_search.h"

namespace okt {

__global__ __launch_bounds__(256) void partition_kernel(
    const uint32_t* __restrict__ idx, const uint64_t* __restrict__ d_nnz, uint64_t n, uint32_t R,
    uint32_t* __restrict__ bounds, uint64_t* __restrict__ offsets) {
    const uint64_t nnz = *d_nnz;
    for (uint64_t r = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; r <= R;
         r += (uint64_t)gridDim.x * blockDim.x) {
        const PartitionCut cut = partition_cut(idx, nnz, n, R, r);
        bounds[r] = cut.bound;
        offsets[r] = cut.offset;
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
