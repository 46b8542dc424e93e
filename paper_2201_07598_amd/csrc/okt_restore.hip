// okt_index_intersect_restore: indexes = local top-k indexes intersected with the
// global top-k indexes (Algorithm 1, line 14), and the residual update
// eps = acc - acc(indexes) (Algorithm 2, line 6) completed on a residual whose
// locally selected entries were zeroed by the select: the locally selected
// entries that did not reach the global top-k are put back.
//
// Work proportional to the local list (about k entries), far below the dense
// passes of an iteration.  A workgroup takes a tile of consecutive local entries;
// because both lists ascend, everything the tile can match lies in one window of
// the global list, found by two binary searches per tile; each entry is then
// searched in that window only.  The matched indices are written in ascending
// order at a position taken from the chained scan over tile counts.
#include "okt_device.h"
#include "okt_sizes.h"

namespace okt {

// First position in a[lo, hi) whose value is >= x.
__device__ __forceinline__ uint32_t lower_bound_u32(const uint32_t* __restrict__ a, uint32_t lo,
                                                    uint32_t hi, uint32_t x) {
    while (lo < hi) {
        const uint32_t mid = lo + ((hi - lo) >> 1);
        if (a[mid] < x) lo = mid + 1; else hi = mid;
    }
    return lo;
}

__global__ __launch_bounds__(RST_BLOCK) void intersect_restore_kernel(
    float* __restrict__ residual, uint32_t n, const uint32_t* __restrict__ local_idx,
    const float* __restrict__ local_val, const uint64_t* __restrict__ d_local_nnz,
    uint32_t max_local, const uint32_t* __restrict__ global_idx,
    const uint64_t* __restrict__ d_global_nnz, uint32_t max_global,
    uint32_t* __restrict__ indexes_out, uint64_t* __restrict__ count_out, ScanHeader* hdr,
    uint64_t* tile_desc, uint64_t* group_desc, uint32_t ntiles) {
    constexpr int WAVES = RST_BLOCK / WAVE;
    __shared__ uint32_t s_tile;
    __shared__ uint32_t s_window[2];
    __shared__ uint32_t s_count[RST_ROWS][WAVES];
    __shared__ uint32_t s_before[2];
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid >> 6;

    if (tid == 0) s_tile = atomicAdd(&hdr->ticket, 1u);
    __syncthreads();
    const uint32_t tile = s_tile;
    const uint64_t have_l = *d_local_nnz, have_g = *d_global_nnz;
    const uint32_t nl = have_l < max_local ? (uint32_t)have_l : max_local;
    const uint32_t ng = have_g < max_global ? (uint32_t)have_g : max_global;
    const uint64_t base64 = (uint64_t)tile * RST_TILE;
    const uint32_t base = base64 < nl ? (uint32_t)base64 : nl;
    const uint32_t end = nl - base > RST_TILE ? base + RST_TILE : nl;

    // ---- the window of the global list this tile can match ----
    if (base < end) {
        if (tid == 0) s_window[0] = lower_bound_u32(global_idx, 0, ng, local_idx[base]);
        if (tid == WAVE) {
            const uint32_t last = local_idx[end - 1];
            // first position above `last`; last = 2^32 - 1 cannot be incremented
            s_window[1] = last == 0xffffffffu ? ng : lower_bound_u32(global_idx, 0, ng, last + 1);
        }
    }
    __syncthreads();
    const uint32_t wlo = base < end ? s_window[0] : 0, whi = base < end ? s_window[1] : 0;

    // ---- membership, restore, rank inside the tile ----
    uint32_t idx[RST_ROWS];
    bool member[RST_ROWS];
    uint64_t ballots[RST_ROWS];
#pragma unroll
    for (int c = 0; c < RST_ROWS; ++c) {
        const uint32_t j = base + c * RST_BLOCK + tid;
        member[c] = false;
        idx[c] = 0;
        if (j < end) {
            idx[c] = local_idx[j];
            const uint32_t pos = lower_bound_u32(global_idx, wlo, whi, idx[c]);
            member[c] = pos < whi && global_idx[pos] == idx[c];
            if (!member[c] && idx[c] < n) residual[idx[c]] = local_val[j];
        }
        ballots[c] = __ballot(member[c]);
        if (lane == 0) s_count[c][wave] = (uint32_t)__popcll(ballots[c]);
    }
    __syncthreads();
    uint32_t aggregate = 0, first[RST_ROWS];
#pragma unroll
    for (int c = 0; c < RST_ROWS; ++c) {
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            if (w == wave) first[c] = aggregate;
            aggregate += s_count[c][w];
        }
    }

    // ---- position of the tile in the output: two waves, two levels, at once ----
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

    if (indexes_out) {
#pragma unroll
        for (int c = 0; c < RST_ROWS; ++c) {
            if (member[c]) {
                const uint64_t m = ballots[c];
                const uint32_t rank = __builtin_amdgcn_mbcnt_hi(
                    (uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
                indexes_out[exclusive + first[c] + rank] = idx[c];
            }
        }
    }
    if (tile == ntiles - 1 && tid == 0) {
        const bool failed =
            __hip_atomic_load(&hdr->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0;
        count_out[0] = failed ? ~0ull : (uint64_t)exclusive + aggregate;
    }
}

}  // namespace okt

extern "C" int okt_index_intersect_restore(
    float* d_residual_inout, uint64_t n, const uint32_t* d_local_idx, const float* d_local_val,
    const uint64_t* d_local_nnz, uint64_t max_local, const uint32_t* d_global_idx,
    const uint64_t* d_global_nnz, uint64_t max_global, uint32_t* d_indexes_out_or_null,
    uint64_t* d_count_out, void* d_ws, size_t ws_bytes, void* stream) {
    using namespace okt;
    hipStream_t s = (hipStream_t)stream;
    if (!d_count_out || !aligned(d_count_out, 8)) return OKT_ERR_INVALID_ARG;
    if (n > 0xffffffffull || max_local > 0xffffffffull || max_global > 0xffffffffull)
        return OKT_ERR_INVALID_ARG;
    if (!d_local_nnz || !d_global_nnz || !aligned(d_local_nnz, 8) || !aligned(d_global_nnz, 8))
        return OKT_ERR_INVALID_ARG;
    if (max_local > 0 && (!d_residual_inout || !d_local_idx || !d_local_val ||
                          !aligned(d_residual_inout, 4) || !aligned(d_local_idx, 4) ||
                          !aligned(d_local_val, 4)))
        return OKT_ERR_INVALID_ARG;
    if (max_global > 0 && (!d_global_idx || !aligned(d_global_idx, 4))) return OKT_ERR_INVALID_ARG;
    if (d_indexes_out_or_null && !aligned(d_indexes_out_or_null, 4)) return OKT_ERR_INVALID_ARG;
    const uint32_t ntiles = (uint32_t)restore_tiles(max_local);
    if (!d_ws || !aligned(d_ws, 256) || ws_bytes < restore_ws_bytes(max_local))
        return OKT_ERR_WORKSPACE;
    ScanHeader* hdr = (ScanHeader*)d_ws;
    uint64_t* tile_desc = (uint64_t*)((char*)d_ws + SCAN_HEADER_BYTES);
    uint64_t* group_desc = tile_desc + ntiles;
    if (launch_zero_words(d_ws, scan_ws_bytes(ntiles) / 8, s) != hipSuccess) return OKT_ERR_HIP;
    hipLaunchKernelGGL(intersect_restore_kernel, dim3(ntiles), dim3(RST_BLOCK), 0, s,
                       d_residual_inout, (uint32_t)n, d_local_idx, d_local_val, d_local_nnz,
                       (uint32_t)max_local, d_global_idx, d_global_nnz, (uint32_t)max_global,
                       d_indexes_out_or_null, d_count_out, hdr, tile_desc, group_desc, ntiles);
    return launch_status();
}
