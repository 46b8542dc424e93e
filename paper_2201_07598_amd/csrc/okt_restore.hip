// okt_index_intersect_restore / okt_index_intersect_zero: indexes = local top-k
// indexes intersected with the global top-k indexes (Algorithm 1, line 14), and
// the residual update eps = acc - acc(indexes) (Algorithm 2, line 6), either
// completed on a residual whose locally selected entries were all zeroed by the
// select (the entries that did not reach the global top-k are put back) or
// applied to the untouched accumulator (the entries of the intersection are
// zeroed).
//
// Work proportional to the local list (about k entries), far below the dense
// passes of an iteration.  A workgroup takes a tile of consecutive local entries;
// because both lists ascend, everything the tile can match lies in one window of
// the global list, whose ends two waves find with a 64-ary search; the window is
// staged in LDS (if it fits) and each entry is searched in it.  The matched
// indices are written in ascending order at a position taken from the chained
// scan over tile counts.
#include "okt_device.h"
#include "okt_sizes.h"

namespace okt {

// First position in a[lo, hi) whose value is >= x, found by one full wave: every
// step probes 64 evenly spaced positions at once, so a list of G entries takes
// about log64(G) dependent memory round trips instead of log2(G).
__device__ __forceinline__ uint32_t wave_lower_bound(const uint32_t* __restrict__ a, uint32_t lo,
                                                     uint32_t hi, uint32_t x) {
    const uint32_t lane = (uint32_t)lane_id();
    while (hi - lo > (uint32_t)WAVE) {
        const uint32_t step = (hi - lo + WAVE - 1) / WAVE;          // >= 2
        const uint64_t at = (uint64_t)lo + (uint64_t)lane * step;   // ascending in the lane
        const bool below = at < hi && a[at] < x;
        const uint32_t c = (uint32_t)__popcll(__ballot(below));     // probes below x: lanes 0..c-1
        if (c == 0) return lo;                                      // a[lo] >= x
        const uint64_t next = (uint64_t)lo + (uint64_t)c * step;    // first probe not below x
        lo = lo + (c - 1) * step + 1;
        if (next < hi) hi = (uint32_t)next;
    }
    const uint64_t at = (uint64_t)lo + lane;
    const bool below = at < hi && a[at] < x;
    return lo + (uint32_t)__popcll(__ballot(below));
}

// Lower bounds of ROWS values in one ascending list, the searches interleaved so
// that their loads overlap.  `at(i)` reads position i of the list.
template <int ROWS, typename At>
__device__ __forceinline__ void lower_bounds(At&& at, uint32_t lo, uint32_t hi,
                                             const uint32_t (&x)[ROWS], const bool (&active)[ROWS],
                                             uint32_t (&pos)[ROWS]) {
    uint32_t len[ROWS];
#pragma unroll
    for (int c = 0; c < ROWS; ++c) {
        pos[c] = lo;
        len[c] = active[c] ? hi - lo : 0;
    }
    for (;;) {
        bool busy = false;
#pragma unroll
        for (int c = 0; c < ROWS; ++c) busy |= len[c] != 0;
        if (!busy) break;
#pragma unroll
        for (int c = 0; c < ROWS; ++c) {
            if (len[c] != 0) {
                const uint32_t half = len[c] >> 1;
                const bool below = at(pos[c] + half) < x[c];
                pos[c] = below ? pos[c] + half + 1 : pos[c];
                len[c] = below ? len[c] - half - 1 : half;
            }
        }
    }
}

// ZERO_MEMBERS false: the vector has every local entry zeroed already, the entries
// outside the intersection get their value back.  true: the vector is the
// untouched accumulator, the entries of the intersection are zeroed (local_val
// is not read).
template <bool ZERO_MEMBERS>
__global__ __launch_bounds__(RST_BLOCK) void intersect_kernel(
    float* __restrict__ residual, uint32_t n, const uint32_t* __restrict__ local_idx,
    const float* __restrict__ local_val, const uint64_t* __restrict__ d_local_nnz,
    uint32_t max_local, const uint32_t* __restrict__ global_idx,
    const uint64_t* __restrict__ d_global_nnz, uint32_t max_global,
    uint32_t* __restrict__ indexes_out, uint64_t* __restrict__ count_out, ScanHeader* hdr,
    uint64_t* tile_desc, uint64_t* group_desc, uint32_t ntiles) {
    constexpr int WAVES = RST_BLOCK / WAVE;
    __shared__ uint32_t s_tile;
    __shared__ uint32_t s_bounds[2];
    __shared__ uint32_t s_count[RST_ROWS][WAVES];
    __shared__ uint32_t s_before[2];
    __shared__ uint32_t s_window[RST_WINDOW];
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

    // ---- the tile's entries, and the window of the global list they can match ----
    uint32_t idx[RST_ROWS];
    bool active[RST_ROWS];
#pragma unroll
    for (int c = 0; c < RST_ROWS; ++c) {
        const uint32_t j = base + c * RST_BLOCK + tid;
        active[c] = j < end;
        idx[c] = active[c] ? local_idx[j] : 0u;
    }
    if (base < end) {                                   // workgroup-uniform
        if (wave == 0) {
            const uint32_t at = wave_lower_bound(global_idx, 0, ng, local_idx[base]);
            if (lane == 0) s_bounds[0] = at;
        } else if (wave == 1) {
            const uint32_t last = local_idx[end - 1];
            // first position above `last`; last = 2^32 - 1 cannot be incremented
            const uint32_t at = last == 0xffffffffu ? ng : wave_lower_bound(global_idx, 0, ng, last + 1);
            if (lane == 0) s_bounds[1] = at;
        }
    }
    __syncthreads();
    const uint32_t wlo = base < end ? s_bounds[0] : 0;
    uint32_t whi = base < end ? s_bounds[1] : 0;
    if (whi < wlo) whi = wlo;                           // only if the local list does not ascend
    const bool staged = whi - wlo <= RST_WINDOW;        // else: search in device memory
    if (staged) {
        for (uint32_t i = tid; i < whi - wlo; i += RST_BLOCK) s_window[i] = global_idx[wlo + i];
        __syncthreads();
    }

    // ---- membership, restore, rank inside the tile ----
    uint32_t pos[RST_ROWS];
    bool member[RST_ROWS];
    uint64_t ballots[RST_ROWS];
    if (staged) {
        lower_bounds<RST_ROWS>([&](uint32_t i) { return s_window[i - wlo]; }, wlo, whi, idx, active, pos);
    } else {
        lower_bounds<RST_ROWS>([&](uint32_t i) { return global_idx[i]; }, wlo, whi, idx, active, pos);
    }
#pragma unroll
    for (int c = 0; c < RST_ROWS; ++c) {
        member[c] = false;
        if (active[c]) {
            if (pos[c] < whi)
                member[c] = (staged ? s_window[pos[c] - wlo] : global_idx[pos[c]]) == idx[c];
            if (ZERO_MEMBERS) {
                if (member[c] && idx[c] < n) residual[idx[c]] = 0.0f;
            } else {
                if (!member[c] && idx[c] < n)
                    residual[idx[c]] = local_val[base + c * RST_BLOCK + tid];
            }
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

namespace okt {

template <bool ZERO_MEMBERS>
static int launch_intersect(float* d_vec, uint64_t n, const uint32_t* d_local_idx,
                            const float* d_local_val, const uint64_t* d_local_nnz,
                            uint64_t max_local, const uint32_t* d_global_idx,
                            const uint64_t* d_global_nnz, uint64_t max_global,
                            uint32_t* d_indexes_out_or_null, uint64_t* d_count_out, void* d_ws,
                            size_t ws_bytes, hipStream_t s) {
    if (!d_count_out || !aligned(d_count_out, 8)) return OKT_ERR_INVALID_ARG;
    if (n > 0xffffffffull || max_local > 0xffffffffull || max_global > 0xffffffffull)
        return OKT_ERR_INVALID_ARG;
    if (!d_local_nnz || !d_global_nnz || !aligned(d_local_nnz, 8) || !aligned(d_global_nnz, 8))
        return OKT_ERR_INVALID_ARG;
    if (max_local > 0 && (!d_vec || !d_local_idx || !aligned(d_vec, 4) || !aligned(d_local_idx, 4)))
        return OKT_ERR_INVALID_ARG;
    if (max_local > 0 && !ZERO_MEMBERS && (!d_local_val || !aligned(d_local_val, 4)))
        return OKT_ERR_INVALID_ARG;
    if (max_global > 0 && (!d_global_idx || !aligned(d_global_idx, 4))) return OKT_ERR_INVALID_ARG;
    if (d_indexes_out_or_null && !aligned(d_indexes_out_or_null, 4)) return OKT_ERR_INVALID_ARG;
    const uint32_t ntiles = (uint32_t)restore_tiles(max_local);
    if (!d_ws || !aligned(d_ws, 256) || ws_bytes < restore_ws_bytes(max_local))
        return OKT_ERR_WORKSPACE;
    ScanHeader* hdr = (ScanHeader*)d_ws;
    uint64_t* tile_desc = (uint64_t*)((char*)d_ws + SCAN_HEADER_BYTES);
    uint64_t* group_desc = tile_desc + ntiles;
    if (launch_clear_scan_state(d_ws, scan_ws_bytes(ntiles) / 8, s) != hipSuccess) return OKT_ERR_HIP;
    timing_before(s);
    hipLaunchKernelGGL(intersect_kernel<ZERO_MEMBERS>, dim3(ntiles), dim3(RST_BLOCK), 0, s, d_vec,
                       (uint32_t)n, d_local_idx, d_local_val, d_local_nnz, (uint32_t)max_local,
                       d_global_idx, d_global_nnz, (uint32_t)max_global, d_indexes_out_or_null,
                       d_count_out, hdr, tile_desc, group_desc, ntiles);
    timing_after(s);
    return launch_status();
}

}  // namespace okt

extern "C" int okt_index_intersect_restore(
    float* d_residual_inout, uint64_t n, const uint32_t* d_local_idx, const float* d_local_val,
    const uint64_t* d_local_nnz, uint64_t max_local, const uint32_t* d_global_idx,
    const uint64_t* d_global_nnz, uint64_t max_global, uint32_t* d_indexes_out_or_null,
    uint64_t* d_count_out, void* d_ws, size_t ws_bytes, void* stream) {
    return okt::launch_intersect<false>(d_residual_inout, n, d_local_idx, d_local_val, d_local_nnz,
                                        max_local, d_global_idx, d_global_nnz, max_global,
                                        d_indexes_out_or_null, d_count_out, d_ws, ws_bytes,
                                        (hipStream_t)stream);
}

extern "C" int okt_index_intersect_zero(
    float* d_acc_inout, uint64_t n, const uint32_t* d_local_idx, const uint64_t* d_local_nnz,
    uint64_t max_local, const uint32_t* d_global_idx, const uint64_t* d_global_nnz,
    uint64_t max_global, uint32_t* d_indexes_out_or_null, uint64_t* d_count_out, void* d_ws,
    size_t ws_bytes, void* stream) {
    return okt::launch_intersect<true>(d_acc_inout, n, d_local_idx, nullptr, d_local_nnz, max_local,
                                       d_global_idx, d_global_nnz, max_global,
                                       d_indexes_out_or_null, d_count_out, d_ws, ws_bytes,
                                       (hipStream_t)stream);
}
