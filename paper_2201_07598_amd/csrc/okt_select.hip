// okt_threshold_select: threshold top-k selection, packaging into a consecutive
// sorted COO buffer, and zeroing of the selected residual entries, in ONE pass
// over acc (Sec. 3.1.3 threshold selection; Sec. 3.1.2 packaging; Algorithm 2,
// line 6 residual update).
//
// HBM-bound: 4 B read per element plus 12 B per selected entry (index, value,
// zero).  A workgroup owns a tile of SEL_TILE consecutive elements, loaded as
// SEL_ITERS float4 per thread with a wave reading 1 KiB contiguous per
// instruction.  Ascending output order inside the tile is (load round, thread,
// component); the ranks come from one packed wave scan (four 16-bit counters in
// a 64-bit word) plus a 16-entry table in LDS.  The position of the tile in the
// output comes from a chained scan over tile counts (decoupled look-back), so
// acc is never read twice.
#include "okt_device.h"
#include "okt_sizes.h"

namespace okt {

static_assert(SEL_ITERS == 4, "the packed scan holds four 16-bit counters");
constexpr int SEL_WAVES = SEL_BLOCK / WAVE;

__global__ __launch_bounds__(SEL_BLOCK) void select_kernel(
    float* __restrict__ acc, uint32_t n, const float* __restrict__ d_threshold,
    uint32_t* __restrict__ idx_out, float* __restrict__ val_out, uint64_t capacity,
    uint64_t* __restrict__ nnz_out, uint32_t* ticket, uint64_t* desc, uint32_t ntiles) {
    __shared__ uint32_t s_tile;
    __shared__ uint32_t s_exclusive;
    __shared__ uint64_t s_wave_total[SEL_WAVES];

    const int tid = threadIdx.x;
    if (tid == 0) s_tile = atomicAdd(ticket, 1u);
    const uint32_t th_key = magnitude_key(*d_threshold);
    __syncthreads();
    const uint32_t tile = s_tile;
    const uint32_t base = tile * (uint32_t)SEL_TILE;     // < n < 2^32

    // ---- load the tile and compare ----
    float4 v[SEL_ITERS];
    uint32_t mask[SEL_ITERS];
    const bool full = (uint64_t)base + SEL_TILE <= n;
    if (full) {
        const float4* src = reinterpret_cast<const float4*>(acc + base);
#pragma unroll
        for (int it = 0; it < SEL_ITERS; ++it) v[it] = src[it * SEL_BLOCK + tid];
#pragma unroll
        for (int it = 0; it < SEL_ITERS; ++it) {
            mask[it] = (magnitude_key(v[it].x) >= th_key ? 1u : 0u) |
                       (magnitude_key(v[it].y) >= th_key ? 2u : 0u) |
                       (magnitude_key(v[it].z) >= th_key ? 4u : 0u) |
                       (magnitude_key(v[it].w) >= th_key ? 8u : 0u);
        }
    } else {
#pragma unroll
        for (int it = 0; it < SEL_ITERS; ++it) {
            const uint64_t i = (uint64_t)base + (uint32_t)(it * SEL_BLOCK + tid) * 4u;
            float e[4];
            uint32_t m = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const bool inside = i + c < n;
                e[c] = inside ? acc[i + c] : 0.0f;
                if (inside && magnitude_key(e[c]) >= th_key) m |= 1u << c;
            }
            v[it] = make_float4(e[0], e[1], e[2], e[3]);
            mask[it] = m;
        }
    }

    // ---- rank inside the tile ----
    uint64_t packed = 0;
#pragma unroll
    for (int it = 0; it < SEL_ITERS; ++it) packed |= (uint64_t)__popc(mask[it]) << (16 * it);
    const uint64_t scan = wave_inclusive_scan<uint64_t>(packed);   // each field <= 256
    const int lane = tid & (WAVE - 1), wave = tid >> 6;
    if (lane == WAVE - 1) s_wave_total[wave] = scan;
    __syncthreads();
    uint32_t round_base[SEL_ITERS];      // first rank of (round it, this wave)
    uint32_t running = 0;
#pragma unroll
    for (int it = 0; it < SEL_ITERS; ++it) {
        uint32_t mine = 0;
#pragma unroll
        for (int w = 0; w < SEL_WAVES; ++w) {
            const uint32_t c = (uint32_t)(s_wave_total[w] >> (16 * it)) & 0xffffu;
            if (w == wave) mine = running;
            running += c;
        }
        round_base[it] = mine;
    }
    const uint32_t aggregate = running;

    // ---- position of the tile in the output ----
    if (wave == 0) {
        const uint32_t ex = lookback_exclusive(desc, tile, aggregate);
        if (lane == 0) s_exclusive = ex;
    }
    __syncthreads();
    const uint32_t exclusive = s_exclusive;

    // ---- emit, in ascending index order, and zero what was emitted ----
    if (aggregate != 0) {
#pragma unroll
        for (int it = 0; it < SEL_ITERS; ++it) {
            const uint32_t m = mask[it];
            if (m == 0) continue;
            const uint32_t incl = (uint32_t)(scan >> (16 * it)) & 0xffffu;
            uint64_t pos = (uint64_t)exclusive + round_base[it] + (incl - __popc(m));
            const uint32_t i0 = base + (uint32_t)(it * SEL_BLOCK + tid) * 4u;
            const float e[4] = {v[it].x, v[it].y, v[it].z, v[it].w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (m & (1u << c)) {
                    if (pos < capacity) {
                        idx_out[pos] = i0 + c;
                        val_out[pos] = e[c];
                        acc[i0 + c] = 0.0f;
                    }
                    ++pos;
                }
            }
        }
    }
    if (tile == ntiles - 1 && tid == 0) {
        const uint64_t total = (uint64_t)exclusive + aggregate;
        nnz_out[0] = total < capacity ? total : capacity;
        nnz_out[1] = total;
    }
}

__global__ void select_empty_kernel(uint64_t* nnz_out) {
    nnz_out[0] = 0;
    nnz_out[1] = 0;
}

}  // namespace okt

extern "C" int okt_threshold_select(float* d_acc_inout, uint64_t n, const float* d_threshold,
                                    uint32_t* d_idx_out, float* d_val_out, uint64_t capacity,
                                    uint64_t* d_nnz_out, void* d_ws, size_t ws_bytes,
                                    void* stream) {
    using namespace okt;
    hipStream_t s = (hipStream_t)stream;
    if (!d_nnz_out || !aligned(d_nnz_out, 8)) return OKT_ERR_INVALID_ARG;
    if (n > 0xffffffffull) return OKT_ERR_INVALID_ARG;
    if (n == 0) {
        hipLaunchKernelGGL(select_empty_kernel, dim3(1), dim3(1), 0, s, d_nnz_out);
        return hipGetLastError() == hipSuccess ? OKT_OK : OKT_ERR_HIP;
    }
    if (!d_acc_inout || !d_threshold || !aligned(d_acc_inout, 16) || !aligned(d_threshold, 4))
        return OKT_ERR_INVALID_ARG;
    if (capacity > 0 && (!d_idx_out || !d_val_out || !aligned(d_idx_out, 4) ||
                         !aligned(d_val_out, 4)))
        return OKT_ERR_INVALID_ARG;
    const uint64_t ntiles = select_tiles(n);
    if (!d_ws || !aligned(d_ws, 256) || ws_bytes < select_ws_bytes(n)) return OKT_ERR_WORKSPACE;
    uint32_t* ticket = (uint32_t*)d_ws;
    uint64_t* desc = (uint64_t*)((char*)d_ws + SCAN_HEADER_BYTES);
    if (launch_zero_words(d_ws, SCAN_HEADER_BYTES / 8 + ntiles, s) != hipSuccess)
        return OKT_ERR_HIP;
    hipLaunchKernelGGL(select_kernel, dim3((unsigned)ntiles), dim3(SEL_BLOCK), 0, s, d_acc_inout,
                       (uint32_t)n, d_threshold, d_idx_out, d_val_out, capacity, d_nnz_out,
                       ticket, desc, (uint32_t)ntiles);
    return hipGetLastError() == hipSuccess ? OKT_OK : OKT_ERR_HIP;
}
