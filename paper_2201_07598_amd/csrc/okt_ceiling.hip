// okt_stream_copy, okt_stream_sum: plain streaming kernels that do none of the
// method's work.  A benchmark times them beside the hot path to know what a
// kernel that only moves bytes reaches on the chip it runs on: the copy for a
// step that reads and writes (accumulate, 8 B in + 4 B out per element), the sum
// for a step that only reads (select at low density, the threshold passes).
#include "okt_device.h"
#include "okt_sizes.h"

namespace okt {

constexpr int CEIL_BLOCK = 256;
constexpr int CEIL_ITERS = 4;
constexpr int CEIL_TILE4 = CEIL_BLOCK * CEIL_ITERS;       // float4 per workgroup and trip
constexpr uint32_t CEIL_SUM_GROUPS = OKT_STREAM_SUM_PARTIALS;

// Like the hot path's kernels, the copy reads and writes a vector far larger than
// the last-level cache with the non-temporal hint (NT, set by the host).
template <bool NT>
__global__ __launch_bounds__(CEIL_BLOCK) void stream_copy_kernel(
    const float* __restrict__ src, float* __restrict__ dst, uint32_t n) {
    const uint32_t n4 = n >> 2;
    const uint32_t base4 = blockIdx.x * (uint32_t)CEIL_TILE4;
    const float4* s4 = reinterpret_cast<const float4*>(src);
    float4* d4 = reinterpret_cast<float4*>(dst);
    if (base4 + CEIL_TILE4 <= n4) {
        float4 v[CEIL_ITERS];
#pragma unroll
        for (int it = 0; it < CEIL_ITERS; ++it)
            v[it] = load_quad<NT>(s4 + base4 + it * CEIL_BLOCK + threadIdx.x);
#pragma unroll
        for (int it = 0; it < CEIL_ITERS; ++it)
            store_quad<NT>(d4 + base4 + it * CEIL_BLOCK + threadIdx.x, v[it]);
        return;
    }
    for (int it = 0; it < CEIL_ITERS; ++it) {
        const uint32_t i = base4 + it * CEIL_BLOCK + threadIdx.x;
        if (i < n4) d4[i] = s4[i];
    }
    const uint32_t tail = (n4 << 2) + threadIdx.x;
    if (threadIdx.x < 4 && tail < n) dst[tail] = src[tail];
}

// The read-only kernel always loads with the non-temporal hint (5 % faster on
// data that is in no cache, which is how it is timed).
__device__ __forceinline__ float4 load_once(const float4* p) { return load_quad<true>(p); }

// Every workgroup strides over the vector, CEIL_ITERS 16-byte loads in flight per
// thread, and leaves one partial sum; nothing else is written.
__global__ __launch_bounds__(CEIL_BLOCK) void stream_sum_kernel(
    const float* __restrict__ src, uint32_t n, float* __restrict__ partials) {
    __shared__ float s_wave[CEIL_BLOCK / 64];
    const uint32_t n4 = n >> 2;
    const float4* s4 = reinterpret_cast<const float4*>(src);
    float sum = 0.f;
    const uint32_t stride4 = gridDim.x * (uint32_t)CEIL_TILE4;
    // trips = ceil(n4 / stride4) for every workgroup: the loop bound is uniform
    for (uint64_t base4 = (uint64_t)blockIdx.x * CEIL_TILE4; base4 < n4; base4 += stride4) {
        float4 v[CEIL_ITERS];
#pragma unroll
        for (int it = 0; it < CEIL_ITERS; ++it) {
            const uint64_t i = base4 + (uint64_t)it * CEIL_BLOCK + threadIdx.x;
            v[it] = i < n4 ? load_once(s4 + i) : float4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int it = 0; it < CEIL_ITERS; ++it) sum += (v[it].x + v[it].y) + (v[it].z + v[it].w);
    }
    if (blockIdx.x == 0 && threadIdx.x < 4) {
        const uint32_t tail = (n4 << 2) + threadIdx.x;
        if (tail < n) sum += src[tail];
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d, 64);
    if ((threadIdx.x & 63) == 0) s_wave[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < CEIL_BLOCK / 64; ++w) t += s_wave[w];
        partials[blockIdx.x] = t;
    }
}

// The memory traffic of the batched sparse reduce without its arithmetic.  Same
// launch shape (one 512-thread workgroup per tile, grid = tiles x regions) and the
// same slice table, so the same pieces of the same arrays are read by the same
// number of waves, in the same way: the slice starts and lengths of up to 256
// contributions are staged in LDS, slice q goes to wave q mod 8, a wave reads a
// slice 64 consecutive entries at a time and keeps ten such blocks, across its
// slices, in flight, index and value together; every entry is then written to the
// output at the place it has in its region's input.  No accumulators, no bitmap,
// no ticket, no scan: what is left is what the gather of these short sorted runs,
// and the write of as many entries, costs on the chip.
__global__ __launch_bounds__(512) void gather_ceiling_kernel(
    const uint32_t* __restrict__ idx_cat, const float* __restrict__ val_cat,
    const uint64_t* __restrict__ seg_begin, uint32_t seg_stride, const uint32_t* __restrict__ lo_hi,
    uint32_t P, uint32_t max_width, uint32_t slots, uint32_t* __restrict__ idx_out,
    float* __restrict__ val_out, uint64_t capacity, const char* __restrict__ ws,
    uint32_t ws_region_bytes, uint32_t table_offset) {
    constexpr int CHUNK = 256, UNITS = 10, WAVES = 8;
    __shared__ uint64_t s_start[CHUNK];
    __shared__ uint32_t s_len[CHUNK];
    const uint32_t region = blockIdx.y, tile = blockIdx.x;
    const uint32_t lo = lo_hi[2 * region], hi = lo_hi[2 * region + 1];
    if (hi < lo || hi - lo > max_width) return;
    const uint32_t ntiles = (uint32_t)(((uint64_t)(hi - lo) + slots - 1) / slots);
    if (tile >= ntiles) return;
    const uint32_t* table = (const uint32_t*)(ws + (size_t)region * ws_region_bytes + table_offset);
    const uint32_t* row0 = table + (size_t)tile * P;
    const uint32_t* row1 = row0 + P;
    const uint64_t* off = seg_begin + (size_t)region * seg_stride;
    const uint64_t first = off[0];                         // the region's entries lie back to back
    idx_out += (size_t)region * capacity;
    val_out += (size_t)region * capacity;
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane(tid >> 6);
    for (uint32_t p0 = 0; p0 < P; p0 += CHUNK) {
        const uint32_t np = P - p0 < (uint32_t)CHUNK ? P - p0 : (uint32_t)CHUNK;
        __syncthreads();
        for (uint32_t q = tid; q < np; q += blockDim.x) {
            const uint32_t b = row0[p0 + q], e = row1[p0 + q];
            s_start[q] = off[p0 + q] + b;
            s_len[q] = e > b ? e - b : 0u;
        }
        __syncthreads();
        uint32_t q = wave, o = 0;                          // next block: slice q, from entry o
        while (q < np) {
            uint64_t pos[UNITS];
            uint32_t left[UNITS];
#pragma unroll
            for (int u = 0; u < UNITS; ++u) {
                while (q < np && s_len[q] == 0) q += WAVES;
                const bool have = q < np;
                const uint32_t len = have ? (uint32_t)__builtin_amdgcn_readfirstlane(s_len[q]) : 0u;
                left[u] = have ? len - o : 0u;
                pos[u] = have ? s_start[q] + o + lane : 0;
                if (have) {
                    o += 64u;
                    if (o >= len) { q += WAVES; o = 0; }
                }
            }
            uint32_t index[UNITS];
            float value[UNITS];
#pragma unroll
            for (int u = 0; u < UNITS; ++u) {
                if (lane < left[u]) {
                    index[u] = idx_cat[pos[u]];
                    value[u] = val_cat[pos[u]];
                }
            }
#pragma unroll
            for (int u = 0; u < UNITS; ++u) {
                const uint64_t at = pos[u] - first;
                if (lane < left[u] && at < capacity) {
                    idx_out[at] = index[u];
                    val_out[at] = value[u];
                }
            }
        }
    }
}

}  // namespace okt

extern "C" int okt_stream_copy(const float* d_src, float* d_dst, uint64_t n, void* stream) {
    using namespace okt;
    if (n == 0) return OKT_OK;
    if (!d_src || !d_dst || n > 0xffffffffull) return OKT_ERR_INVALID_ARG;
    if (!aligned(d_src, 16) || !aligned(d_dst, 16)) return OKT_ERR_INVALID_ARG;
    const uint64_t blocks = (n >> 2) / CEIL_TILE4 + 1;     // the last one owns the ragged end
    timing_before((hipStream_t)stream);
    auto* kernel = stream_past_cache(n) ? stream_copy_kernel<true> : stream_copy_kernel<false>;
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(CEIL_BLOCK), 0, (hipStream_t)stream,
                       d_src, d_dst, (uint32_t)n);
    timing_after((hipStream_t)stream);
    return launch_status();
}

extern "C" int okt_stream_sum(const float* d_src, uint64_t n, float* d_partials_out, void* stream) {
    using namespace okt;
    if ((!d_src && n) || !d_partials_out || n > 0xffffffffull) return OKT_ERR_INVALID_ARG;
    if (!aligned(d_src, 16) || !aligned(d_partials_out, 4)) return OKT_ERR_INVALID_ARG;
    timing_before((hipStream_t)stream);
    hipLaunchKernelGGL(stream_sum_kernel, dim3(CEIL_SUM_GROUPS), dim3(CEIL_BLOCK), 0,
                       (hipStream_t)stream, d_src, (uint32_t)n, d_partials_out);
    timing_after((hipStream_t)stream);
    return launch_status();
}
