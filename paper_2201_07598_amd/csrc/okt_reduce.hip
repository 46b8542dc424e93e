// okt_sparse_reduce / okt_sparse_reduce_batch: the local reduction of the P
// sparse contributions a worker receives for its region (Algorithm 1, line 8;
// Sec. 3.1.1).  Plain sum over the union of the supports.
//
// A workgroup owns RED_TILE consecutive index slots of the region.  It finds
// its slice of every contribution by binary search (contributions are sorted),
// then streams the slices, flattened into one list so that all 256 threads stay
// busy whatever the slice lengths, into a dense fp64 tile in LDS (LDS atomic add;
// a bitmap records which slots were hit).  The tile is then compacted in index
// order; its position in the output comes from a chained scan over tile counts.
// Traffic: every input entry is read once (8 B), every output entry written
// once (8 B), plus 4 B per slot if the dense region is requested.
#include "okt_device.h"
#include "okt_sizes.h"

namespace okt {

constexpr int RED_WORDS = RED_TILE / 32;

__device__ __forceinline__ uint64_t lower_bound_idx(const uint32_t* __restrict__ a, uint64_t lo,
                                                    uint64_t hi, uint32_t x) {
    while (lo < hi) {
        const uint64_t mid = lo + ((hi - lo) >> 1);
        if (a[mid] < x) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// grid = (tiles of the widest region, B).  Region j: chunk offsets at
// chunk_off + j*(P+1); bounds from lo_hi[2j..] if lo_hi != NULL else (lo0, hi0).
__global__ __launch_bounds__(RED_BLOCK) void reduce_kernel(
    const uint32_t* __restrict__ idx_cat, const float* __restrict__ val_cat,
    const uint64_t* __restrict__ chunk_off, const uint32_t* __restrict__ lo_hi, uint32_t lo0,
    uint32_t hi0, uint32_t P, uint32_t max_width, uint32_t* __restrict__ idx_out,
    float* __restrict__ val_out, uint64_t capacity, uint64_t* __restrict__ nnz_out,
    float* __restrict__ dense_out, char* ws, uint32_t ws_region_bytes) {
    __shared__ double s_sum[RED_TILE];
    __shared__ uint32_t s_bits[RED_WORDS];
    __shared__ uint64_t s_start[RED_CHUNKS];
    __shared__ uint32_t s_prefix[RED_CHUNKS + 1];
    __shared__ uint32_t s_wave[RED_BLOCK / WAVE];
    __shared__ uint32_t s_tile, s_before[2];

    const int tid = threadIdx.x;
    const uint32_t region = blockIdx.y;
    ScanHeader* hdr = (ScanHeader*)(ws + (size_t)region * ws_region_bytes);
    uint64_t* tile_desc = (uint64_t*)(ws + (size_t)region * ws_region_bytes + SCAN_HEADER_BYTES);
    uint64_t* group_desc = tile_desc + gridDim.x;
    if (tid == 0) s_tile = atomicAdd(&hdr->ticket, 1u);

    const uint32_t lo = lo_hi ? lo_hi[2 * region] : lo0;
    const uint32_t hi = lo_hi ? lo_hi[2 * region + 1] : hi0;
    uint64_t* nnz = nnz_out + 2 * (size_t)region;
    const bool bad = hi < lo || hi - lo > max_width;
    const uint32_t width = bad ? 0u : hi - lo;
    const uint32_t ntiles = (width + RED_TILE - 1) / RED_TILE;

    for (int s = tid; s < RED_TILE; s += RED_BLOCK) s_sum[s] = 0.0;
    if (tid < RED_WORDS) s_bits[tid] = 0;
    __syncthreads();
    const uint32_t tile = s_tile;
    if (ntiles == 0) {
        if (tile == 0 && tid == 0) {
            nnz[0] = bad ? ~0ull : 0ull;
            nnz[1] = bad ? ~0ull : 0ull;
        }
        return;
    }
    if (tile >= ntiles) return;
    const uint32_t a = lo + tile * (uint32_t)RED_TILE;              // first index of the tile
    const uint32_t slots = (hi - a) < (uint32_t)RED_TILE ? (hi - a) : (uint32_t)RED_TILE;
    const uint64_t* off = chunk_off + (size_t)region * (P + 1);
    idx_out += (size_t)region * capacity;
    val_out += (size_t)region * capacity;

    // ---- accumulate the contributions, RED_CHUNKS of them per sweep ----
    for (uint32_t p0 = 0; p0 < P; p0 += RED_CHUNKS) {
        const uint32_t np = (P - p0) < (uint32_t)RED_CHUNKS ? (P - p0) : (uint32_t)RED_CHUNKS;
        // slice of contribution p0+q that falls into [a, a+slots)
        for (uint32_t q = tid; q < np; q += RED_BLOCK) {
            const uint64_t cb = off[p0 + q], ce = off[p0 + q + 1];
            const uint64_t sb = lower_bound_idx(idx_cat, cb, ce, a);
            // a + slots may be 2^32 only if hi is; hi <= 2^32-1, so it fits
            const uint64_t se = lower_bound_idx(idx_cat, sb, ce, a + slots);
            s_start[q] = sb;
            s_prefix[q + 1] = (uint32_t)(se - sb);      // <= RED_TILE
        }
        if (tid == 0) s_prefix[0] = 0;
        __syncthreads();
        // inclusive scan of the np counts (np <= 1024: four per thread)
        {
            uint32_t c[RED_CHUNKS / RED_BLOCK];
            uint32_t sum = 0;
#pragma unroll
            for (int j = 0; j < RED_CHUNKS / RED_BLOCK; ++j) {
                const uint32_t q = tid * (RED_CHUNKS / RED_BLOCK) + j;
                c[j] = q < np ? s_prefix[q + 1] : 0u;
                sum += c[j];
            }
            const uint32_t incl = wave_inclusive_scan<uint32_t>(sum);
            const int lane = tid & (WAVE - 1), wave = tid >> 6;
            if (lane == WAVE - 1) s_wave[wave] = incl;
            __syncthreads();
            uint32_t before = incl - sum;
            for (int w = 0; w < wave; ++w) before += s_wave[w];
#pragma unroll
            for (int j = 0; j < RED_CHUNKS / RED_BLOCK; ++j) {
                const uint32_t q = tid * (RED_CHUNKS / RED_BLOCK) + j;
                before += c[j];
                if (q < np) s_prefix[q + 1] = before;
            }
        }
        __syncthreads();
        const uint32_t total = s_prefix[np];
        for (uint32_t j = tid; j < total; j += RED_BLOCK) {
            // contribution q with s_prefix[q] <= j < s_prefix[q+1]
            uint32_t ql = 0, qh = np;
            while (qh - ql > 1) {
                const uint32_t mid = (ql + qh) >> 1;
                if (s_prefix[mid] <= j) ql = mid; else qh = mid;
            }
            const uint64_t pos = s_start[ql] + (j - s_prefix[ql]);
            const uint32_t slot = idx_cat[pos] - a;
            const double v = (double)val_cat[pos];
            if (slot >= slots) continue;     // only reachable with unsorted input
            __hip_atomic_fetch_add(&s_sum[slot], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            __hip_atomic_fetch_or(&s_bits[slot >> 5], 1u << (slot & 31), __ATOMIC_RELAXED,
                                  __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        __syncthreads();
    }

    // ---- count, chain, compact ----
    const int lane = tid & (WAVE - 1), wave = tid >> 6;
    const uint32_t word = tid < RED_WORDS ? s_bits[tid] : 0u;
    const uint32_t cnt = __popc(word);
    const uint32_t incl = wave_inclusive_scan<uint32_t>(cnt);
    if (lane == WAVE - 1) s_wave[wave] = incl;
    __syncthreads();
    uint32_t rank = incl - cnt, aggregate = 0;
    for (int w = 0; w < RED_BLOCK / WAVE; ++w) {
        if (w < wave) rank += s_wave[w];
        aggregate += s_wave[w];
    }
    const uint32_t group = tile / SCAN_GROUP;
    if (wave == 0) {
        const uint32_t before = scan_within_group(hdr, tile_desc, group_desc, tile, aggregate);
        if (lane == 0) s_before[0] = before;
    } else if (wave == 1) {
        const uint32_t before = scan_across_groups(hdr, group_desc, group);
        if (lane == 0) s_before[1] = before;
    }
    __syncthreads();
    const uint32_t exclusive = s_before[0] + s_before[1];
    if (tid == 0 && group != 0 && tile % SCAN_GROUP == SCAN_GROUP - 1)
        scan_close_group(group_desc, group, exclusive + aggregate);
    {
        uint32_t w = word;
        uint64_t pos = (uint64_t)exclusive + rank;
        while (w) {
            const int bit = __ffs(w) - 1;
            w &= w - 1;
            const uint32_t slot = (uint32_t)tid * 32u + bit;
            if (pos < capacity) {
                idx_out[pos] = a + slot;
                val_out[pos] = (float)s_sum[slot];
            }
            ++pos;
        }
    }
    if (dense_out) {
        float* dst = dense_out + (size_t)region * max_width + (size_t)tile * RED_TILE;
        for (uint32_t s = tid; s < slots; s += RED_BLOCK) dst[s] = (float)s_sum[s];
    }
    if (tile == ntiles - 1 && tid == 0) {
        const uint64_t total = (uint64_t)exclusive + aggregate;
        const bool failed =
            __hip_atomic_load(&hdr->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0;
        nnz[0] = failed ? ~0ull : (total < capacity ? total : capacity);
        nnz[1] = failed ? ~0ull : total;
    }
}

static int reduce_launch(const uint32_t* d_idx_cat, const float* d_val_cat,
                         const uint64_t* d_chunk_off, const uint32_t* d_lo_hi, uint32_t lo,
                         uint32_t hi, uint32_t B, uint32_t P, uint32_t max_width,
                         uint32_t* d_idx_out, float* d_val_out, uint64_t capacity,
                         uint64_t* d_nnz_out, float* d_dense, void* d_ws, size_t ws_bytes,
                         hipStream_t s) {
    if (!d_idx_cat || !d_val_cat || !d_chunk_off || !d_nnz_out) return OKT_ERR_INVALID_ARG;
    if (P == 0 || P > 65535 || B == 0 || B > 65535) return OKT_ERR_INVALID_ARG;
    if (capacity > 0 && (!d_idx_out || !d_val_out)) return OKT_ERR_INVALID_ARG;
    if (!aligned(d_idx_cat, 4) || !aligned(d_val_cat, 4) || !aligned(d_chunk_off, 8) ||
        !aligned(d_nnz_out, 8) || !aligned(d_idx_out, 4) || !aligned(d_val_out, 4) ||
        !aligned(d_dense, 4) || !aligned(d_lo_hi, 4))
        return OKT_ERR_INVALID_ARG;
    const size_t region_bytes = reduce_ws_bytes_region(max_width);
    if (!d_ws || !aligned(d_ws, 256) || ws_bytes < region_bytes * B) return OKT_ERR_WORKSPACE;
    uint64_t tiles = reduce_tiles(max_width);
    if (tiles == 0) tiles = 1;
    if (launch_zero_words(d_ws, region_bytes * B / 8, s) != hipSuccess) return OKT_ERR_HIP;
    hipLaunchKernelGGL(reduce_kernel, dim3((unsigned)tiles, B), dim3(RED_BLOCK), 0, s, d_idx_cat,
                       d_val_cat, d_chunk_off, d_lo_hi, lo, hi, P, max_width, d_idx_out,
                       d_val_out, capacity, d_nnz_out, d_dense, (char*)d_ws,
                       (uint32_t)region_bytes);
    return hipGetLastError() == hipSuccess ? OKT_OK : OKT_ERR_HIP;
}

}  // namespace okt

extern "C" int okt_sparse_reduce(const uint32_t* d_idx_cat, const float* d_val_cat,
                                 const uint64_t* d_chunk_off, uint32_t P, uint32_t lo, uint32_t hi,
                                 uint32_t* d_idx_out, float* d_val_out, uint64_t capacity,
                                 uint64_t* d_nnz_out, float* d_dense_out_or_null, void* d_ws,
                                 size_t ws_bytes, void* stream) {
    if (lo > hi) return OKT_ERR_INVALID_ARG;
    return okt::reduce_launch(d_idx_cat, d_val_cat, d_chunk_off, nullptr, lo, hi, 1, P, hi - lo,
                              d_idx_out, d_val_out, capacity, d_nnz_out, d_dense_out_or_null,
                              d_ws, ws_bytes, (hipStream_t)stream);
}

extern "C" int okt_sparse_reduce_batch(const uint32_t* d_idx_cat, const float* d_val_cat,
                                       const uint64_t* d_chunk_off, const uint32_t* d_lo_hi,
                                       uint32_t B, uint32_t P, uint32_t max_width,
                                       uint32_t* d_idx_out, float* d_val_out, uint64_t capacity,
                                       uint64_t* d_nnz_out, float* d_dense_out_or_null,
                                       void* d_ws, size_t ws_bytes, void* stream) {
    if (!d_lo_hi) return OKT_ERR_INVALID_ARG;
    return okt::reduce_launch(d_idx_cat, d_val_cat, d_chunk_off, d_lo_hi, 0, 0, B, P, max_width,
                              d_idx_out, d_val_out, capacity, d_nnz_out, d_dense_out_or_null,
                              d_ws, ws_bytes, (hipStream_t)stream);
}
