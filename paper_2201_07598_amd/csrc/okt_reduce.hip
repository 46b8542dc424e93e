// okt_sparse_reduce / okt_sparse_reduce_batch: the local reduction of the P
// sparse contributions a worker receives for its region (Algorithm 1, line 8;
// Sec. 3.1.1).  Plain sum over the union of the supports.
//
// Two kernels per call.
//  1. reduce_slices_kernel: the region is cut into tiles of `slots` consecutive
//     index slots; one thread per (tile boundary, contribution) finds, by binary
//     search in the sorted contribution, where the boundary falls.  All searches
//     of a call run side by side, so their latency is paid once.
//  2. reduce_tile_kernel: a workgroup owns one tile.  Its slice of every
//     contribution is known from the table, so all its entries are addressed up
//     front: the slices go round-robin to the waves, a wave reads a slice 64
//     consecutive entries at a time and keeps several such blocks, across its
//     slices, in flight.  Entries are summed with LDS fp64 atomic adds.  Where the region is densely hit the accumulator of a slot is
//     the slot itself.  Where it is sparsely hit the tile is wider than the
//     accumulator array: a first sweep marks the hit slots in a bitmap, the
//     popcount prefix of the bitmap ranks them, and the second sweep sums into
//     accumulator [rank].  The tile is then written out in index order; its place
//     in the output comes from the two-level chained scan over tile counts.
// Traffic: every input entry is read once from HBM (the second sweep hits in
// cache), every output entry is written once, plus 4 B per slot if the dense
// region is requested.
#include "okt_device.h"
#include "okt_search.h"
#include "okt_sizes.h"

#include <type_traits>

namespace okt {

constexpr int RED_WAVES = RED_BLOCK / WAVE;

struct RegionView {
    uint32_t lo, hi, width, ntiles;
    bool bad;
};
__device__ __forceinline__ RegionView region_view(const uint32_t* lo_hi, uint32_t lo0, uint32_t hi0,
                                                  uint32_t region, uint32_t max_width,
                                                  uint32_t slots) {
    RegionView r;
    r.lo = lo_hi ? lo_hi[2 * region] : lo0;
    r.hi = lo_hi ? lo_hi[2 * region + 1] : hi0;
    r.bad = r.hi < r.lo || r.hi - r.lo > max_width;
    r.width = r.bad ? 0u : r.hi - r.lo;
    r.ntiles = (uint32_t)(((uint64_t)r.width + slots - 1) / slots);
    return r;
}

// table[region][t][p] = number of entries of contribution p with index below
// lo + t * slots (clipped to hi), for t = 0 .. ntiles.
// from_guess: a launch with so many boundaries that it is bound by the number of
// probes, not by the latency of one search, starts every search from a guess.
__global__ __launch_bounds__(256) void reduce_slices_kernel(
    const uint32_t* __restrict__ idx_cat, const uint64_t* __restrict__ seg_begin,
    const uint64_t* __restrict__ seg_end, uint32_t seg_stride,
    const uint32_t* __restrict__ lo_hi, uint32_t lo0, uint32_t hi0, uint32_t P,
    uint32_t max_width, uint32_t slots, char* ws, uint32_t ws_region_bytes,
    uint32_t table_offset, uint32_t spin_limit, uint32_t from_guess) {
    const uint32_t region = blockIdx.y;
    const RegionView r = region_view(lo_hi, lo0, hi0, region, max_width, slots);
    uint32_t* table = (uint32_t*)(ws + (size_t)region * ws_region_bytes + table_offset);
    // the scan state of the region (header and descriptors, in front of the table)
    // must be zero when the tile kernel starts
    uint64_t* scan_state = (uint64_t*)(ws + (size_t)region * ws_region_bytes);
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < table_offset / 8;
         i += gridDim.x * blockDim.x)
        scan_state[i] = i == SCAN_SPIN_WORD ? (uint64_t)spin_limit : 0ull;
    const uint64_t* begin = seg_begin + (size_t)region * seg_stride;
    const uint64_t* end = seg_end + (size_t)region * seg_stride;
    const uint64_t cells = (uint64_t)(r.ntiles + 1) * P;
    for (uint64_t c = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; c < cells;
         c += (uint64_t)gridDim.x * blockDim.x) {
        // neighbouring threads search the same contribution for neighbouring
        // boundaries: their probes share all but the last few levels
        const uint32_t p = (uint32_t)(c / (r.ntiles + 1)), t = (uint32_t)(c % (r.ntiles + 1));
        uint64_t bound = (uint64_t)r.lo + (uint64_t)t * slots;
        if (bound > r.hi) bound = r.hi;
        const uint64_t cb = begin[p], ce = end[p] > cb ? end[p] : cb;
        // where the boundary would fall if the contribution's indices were spread evenly
        // over the region (both factors are below 2^32)
        const uint64_t guess = cb + (r.width ? (ce - cb) * (bound - r.lo) / r.width : 0);
        table[(size_t)t * P + p] =
            (uint32_t)((from_guess ? lower_bound_near(idx_cat, cb, ce, (uint32_t)bound, guess)
                                   : lower_bound_idx(idx_cat, cb, ce, (uint32_t)bound)) - cb);
    }
}

// The same table for launches with few cells (a lone region): one WAVE per cell,
// 64 evenly spaced probes per step, so a boundary is found in about log64 of the
// contribution's length dependent round trips instead of log2 - this kernel is
// nothing but that latency.  (For many regions the extra probes would cost more
// memory traffic than the latency they save.)
__global__ __launch_bounds__(256) void reduce_slices_wave_kernel(
    const uint32_t* __restrict__ idx_cat, const uint64_t* __restrict__ seg_begin,
    const uint64_t* __restrict__ seg_end, uint32_t seg_stride,
    const uint32_t* __restrict__ lo_hi, uint32_t lo0, uint32_t hi0, uint32_t P,
    uint32_t max_width, uint32_t slots, char* ws, uint32_t ws_region_bytes,
    uint32_t table_offset, uint32_t spin_limit) {
    const uint32_t region = blockIdx.y;
    const RegionView r = region_view(lo_hi, lo0, hi0, region, max_width, slots);
    uint32_t* table = (uint32_t*)(ws + (size_t)region * ws_region_bytes + table_offset);
    uint64_t* scan_state = (uint64_t*)(ws + (size_t)region * ws_region_bytes);
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < table_offset / 8;
         i += gridDim.x * blockDim.x)
        scan_state[i] = i == SCAN_SPIN_WORD ? (uint64_t)spin_limit : 0ull;
    const uint64_t* begin = seg_begin + (size_t)region * seg_stride;
    const uint64_t* end = seg_end + (size_t)region * seg_stride;
    const uint64_t cells = (uint64_t)(r.ntiles + 1) * P;
    const uint32_t lane = threadIdx.x & (WAVE - 1);
    const uint64_t waves = (uint64_t)gridDim.x * (blockDim.x / WAVE);
    for (uint64_t c = (uint64_t)blockIdx.x * (blockDim.x / WAVE) + threadIdx.x / WAVE; c < cells;
         c += waves) {
        const uint32_t p = (uint32_t)(c / (r.ntiles + 1)), t = (uint32_t)(c % (r.ntiles + 1));
        uint64_t bound = (uint64_t)r.lo + (uint64_t)t * slots;
        if (bound > r.hi) bound = r.hi;
        const uint32_t x = (uint32_t)bound;                 // bound <= hi < 2^32
        const uint64_t cb = begin[p];
        uint64_t lo = cb, hi = end[p] > cb ? end[p] : cb;   // the answer lies in [lo, hi]
        while (hi - lo > (uint64_t)WAVE) {
            const uint64_t step = (hi - lo + WAVE - 1) / WAVE;
            const uint64_t at = lo + lane * step;
            const bool below = at < hi && idx_cat[at] < x;
            const uint32_t n_below = (uint32_t)__popcll(__ballot(below));   // lanes 0 .. n_below-1
            if (n_below == 0) { hi = lo; break; }                           // idx_cat[lo] >= x
            const uint64_t next = lo + (uint64_t)n_below * step;            // first probe not below x
            lo = lo + (uint64_t)(n_below - 1) * step + 1;
            if (next < hi) hi = next;
        }
        if (hi > lo) {
            const bool below = lo + lane < hi && idx_cat[lo + lane] < x;
            lo += (uint64_t)__popcll(__ballot(below));
        }
        if (lane == 0) table[(size_t)t * P + p] = (uint32_t)(lo - cb);
    }
}

// Exclusive prefix over the popcounts of `words` bitmap words into s_wprefix;
// returns the total (to every thread).  Called by the whole workgroup.
template <uint32_t WORDS_MAX>
__device__ __forceinline__ uint32_t bitmap_prefix(const uint32_t* s_bits, uint16_t* s_wprefix,
                                                  uint32_t words, uint32_t* s_wave) {
    static_assert(WORDS_MAX % RED_BLOCK == 0 || WORDS_MAX < RED_BLOCK,
                  "every thread owns the same number of bitmap words");
    constexpr uint32_t PER = (WORDS_MAX + RED_BLOCK - 1) / RED_BLOCK;   // words per thread (1 to 3)
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid >> 6;
    uint32_t c[PER], sum = 0;
#pragma unroll
    for (uint32_t j = 0; j < PER; ++j) {
        const uint32_t w = tid * PER + j;
        c[j] = w < words ? (uint32_t)__popc(s_bits[w]) : 0u;
        sum += c[j];
    }
    const uint32_t incl = wave_inclusive_scan<uint32_t>(sum);
    if (lane == WAVE - 1) s_wave[wave] = incl;
    __syncthreads();
    uint32_t before = incl - sum, total = 0;
#pragma unroll
    for (int w = 0; w < RED_WAVES; ++w) {
        if (w < wave) before += s_wave[w];
        total += s_wave[w];
    }
#pragma unroll
    for (uint32_t j = 0; j < PER; ++j) {
        const uint32_t w = tid * PER + j;
        if (w < words) s_wprefix[w] = (uint16_t)before;       // < 32 * WORDS_MAX <= 65536
        before += c[j];
    }
    __syncthreads();
    return total;
}

// grid = (tiles of the widest region, B).  Region j: chunk offsets at
// seg_begin / seg_end + j * seg_stride; bounds from lo_hi[2j..] if lo_hi != NULL else
// (lo0, hi0).
// C accumulators, a bitmap of S_MAX slots: (RED_C, RED_S_MAX); (RED_C_SPARSE,
// RED_S_SPARSE) for very sparsely hit regions; (RED_C_DENSE, RED_C_DENSE) for
// densely hit ones, where the accumulator of a slot is the slot itself.
template <uint32_t C, uint32_t S_MAX>
__global__ __launch_bounds__(RED_BLOCK) void reduce_tile_kernel(
    const uint32_t* __restrict__ idx_cat, const float* __restrict__ val_cat,
    const uint64_t* __restrict__ seg_begin, uint32_t seg_stride,
    const uint32_t* __restrict__ lo_hi, uint32_t lo0,
    uint32_t hi0, uint32_t P, uint32_t max_width, uint32_t slots, uint32_t* __restrict__ idx_out,
    float* __restrict__ val_out, uint64_t capacity, uint64_t* __restrict__ nnz_out,
    float* __restrict__ dense_out, char* ws, uint32_t ws_region_bytes, uint32_t table_offset,
    uint32_t span_blocks) {
    constexpr uint32_t WORDS_MAX = S_MAX / 32;
    static_assert(S_MAX <= 65536, "slots and ranks are kept in 16 bits");
    __shared__ double s_sum[C];
    __shared__ uint32_t s_bits[WORDS_MAX];
    __shared__ uint16_t s_wprefix[WORDS_MAX];
    constexpr bool CAN_RANK = S_MAX > C;          // else: accumulator = slot, always
    __shared__ uint16_t s_slot[CAN_RANK ? C : 1]; // ranked tiles: slot of accumulator [rank]
    __shared__ uint64_t s_start[RED_CHUNKS];      // slice starts of the current sweep
    __shared__ uint32_t s_len[RED_CHUNKS];        // slice lengths
    __shared__ uint32_t s_loaded_p0;              // which sweep they belong to
    __shared__ uint32_t s_wave[RED_WAVES];
    __shared__ uint32_t s_tile, s_before[2];

    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid >> 6;
    const uint32_t region = blockIdx.y;
    char* region_ws = ws + (size_t)region * ws_region_bytes;
    ScanHeader* hdr = (ScanHeader*)region_ws;
    uint64_t* tile_desc = (uint64_t*)(region_ws + SCAN_HEADER_BYTES);
    uint64_t* group_desc = tile_desc + gridDim.x;
    const uint32_t* table = (const uint32_t*)(region_ws + table_offset);
    if (tid == 0) {
        s_tile = atomicAdd(&hdr->ticket, 1u);
        s_loaded_p0 = ~0u;
    }

    const RegionView r = region_view(lo_hi, lo0, hi0, region, max_width, slots);
    uint64_t* nnz = nnz_out + 2 * (size_t)region;
    const bool ranked = CAN_RANK && slots > C;   // accumulators indexed by rank, not by slot
    const uint32_t words_all = slots / 32;       // slots is a multiple of 32
    // the bitmap and the accumulators are cleared while the ticket is under way
    for (uint32_t w = tid; w < words_all; w += RED_BLOCK) s_bits[w] = 0;
    for (uint32_t s = tid; s < C; s += RED_BLOCK) s_sum[s] = 0.0;
    __syncthreads();
    const uint32_t tile = s_tile;
    if (r.ntiles == 0) {
        if (tile == 0 && tid == 0) {
            nnz[0] = r.bad ? ~0ull : 0ull;
            nnz[1] = r.bad ? ~0ull : 0ull;
        }
        return;
    }
    if (tile >= r.ntiles) return;
    const uint32_t a = r.lo + tile * slots;                       // first index of the tile
    const uint32_t tslots = (r.hi - a) < slots ? (r.hi - a) : slots;
    const uint32_t words = (tslots + 31) / 32;
    const uint64_t* off = seg_begin + (size_t)region * seg_stride;
    const uint32_t* row0 = table + (size_t)tile * P;              // slice starts
    const uint32_t* row1 = row0 + P;                              // slice ends
    idx_out += (size_t)region * capacity;
    val_out += (size_t)region * capacity;

    // Hands every entry of the tile to body(index, value).  Contributions are
    // taken RED_CHUNKS at a time; slice q of a sweep belongs to wave q mod WAVES,
    // whose lanes read it in spans of G x 64 consecutive entries (G coalesced loads
    // that share one address and one piece of bookkeeping).  A wave first names up
    // to UNITS such spans, across its slices, then issues all their loads, then
    // consumes them: enough loads in flight to cover the memory latency, no
    // per-entry search, and only wave-uniform bookkeeping.  Long slices (few
    // contributions) take G = 4 or 2; short ones G = 1, where a longer span would
    // be mostly empty (the host picks from the expected slice length).
    auto for_each_entry_in = [&](auto with_values, auto span, auto units, auto&& body) {
        constexpr bool VALUES = decltype(with_values)::value;
        constexpr int G = decltype(span)::value, UNITS = decltype(units)::value;
        for (uint32_t p0 = 0; p0 < P; p0 += RED_CHUNKS) {
            const uint32_t np = (P - p0) < (uint32_t)RED_CHUNKS ? (P - p0) : (uint32_t)RED_CHUNKS;
            // Every thread must take the same branch here.  The note of what is
            // loaded is therefore written between the two barriers: each thread has
            // read it (before the first) when it changes, and sees the new value
            // (after the second) when it next looks.  Written after the second
            // barrier instead, a wave that ran ahead could still read the value an
            // earlier sweep left for this very chunk and skip the reload alone.
            if (p0 != s_loaded_p0) {            // slice table of this sweep not in LDS yet
                __syncthreads();
                for (uint32_t q = tid; q < np; q += RED_BLOCK) {
                    const uint32_t b = row0[p0 + q], e = row1[p0 + q];
                    s_start[q] = off[p0 + q] + b;
                    s_len[q] = e > b ? e - b : 0u;      // e < b only for unsorted input
                }
                if (tid == 0) s_loaded_p0 = p0;
                __syncthreads();
            }
            uint32_t q = (uint32_t)__builtin_amdgcn_readfirstlane(wave), o = 0;   // next span: slice q, from entry o
            while (q < np) {
                uint64_t pos[UNITS];
                uint32_t left[UNITS];            // entries of the slice from the span's start on (wave-uniform)
#pragma unroll
                for (int u = 0; u < UNITS; ++u) {
                    // skip empty slices
                    while (q < np && s_len[q] == 0) q += RED_WAVES;
                    const bool have = q < np;
                    const uint32_t len =
                        have ? (uint32_t)__builtin_amdgcn_readfirstlane(s_len[q]) : 0u;
                    left[u] = have ? len - o : 0u;
                    pos[u] = have ? s_start[q] + o + lane : 0;
                    if (have) {
                        o += G * WAVE;
                        if (o >= len) { q += RED_WAVES; o = 0; }
                    }
                }
                uint32_t index[UNITS][G];
                float value[UNITS][G];
#pragma unroll
                for (int u = 0; u < UNITS; ++u) {
#pragma unroll
                    for (int j = 0; j < G; ++j) {
                        if ((uint32_t)lane + (uint32_t)(j * WAVE) < left[u]) {
                            index[u][j] = idx_cat[pos[u] + j * WAVE];
                            if (VALUES) value[u][j] = val_cat[pos[u] + j * WAVE];
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < UNITS; ++u) {
#pragma unroll
                    for (int j = 0; j < G; ++j)
                        if ((uint32_t)lane + (uint32_t)(j * WAVE) < left[u])
                            body(index[u][j], VALUES ? value[u][j] : 0.0f);
                }
            }
        }
    };
    auto for_each_entry = [&](auto with_values, auto&& body) {
        if (span_blocks == 4)
            for_each_entry_in(with_values, std::integral_constant<int, 4>{},
                              std::integral_constant<int, 3>{}, body);
        else if (span_blocks == 2)
            for_each_entry_in(with_values, std::integral_constant<int, 2>{},
                              std::integral_constant<int, 6>{}, body);
        else
            for_each_entry_in(with_values, std::integral_constant<int, 1>{},
                              std::integral_constant<int, RED_UNROLL>{}, body);
    };
    using Yes = std::true_type;      // sweep needs the values too
    using No = std::false_type;      // sweep needs the indices only

    // Both waves of the chained scan; every thread gets the count of all tiles
    // before this one.
    auto place_tile = [&](uint32_t count) -> uint32_t {
        const uint32_t group = tile / SCAN_GROUP;
        if (wave == 0) {
            const uint32_t before = scan_within_group(hdr, tile_desc, group_desc, tile, count);
            if (lane == 0) s_before[0] = before;
        } else if (wave == 1) {
            const uint32_t before = scan_across_groups(hdr, group_desc, group);
            if (lane == 0) s_before[1] = before;
        }
        __syncthreads();
        const uint32_t before = s_before[0] + s_before[1];
        if (tid == 0 && group != 0 && tile % SCAN_GROUP == SCAN_GROUP - 1)
            scan_close_group(group_desc, group, before + count);
        return before;
    };
    float* dense = dense_out ? dense_out + (size_t)region * max_width + (size_t)tile * slots
                             : nullptr;
    uint32_t distinct, exclusive;

    if (!ranked) {
        // ---- densely hit region: accumulator = slot, one sweep ----
        for_each_entry(Yes{}, [&](uint32_t index, float x) {
            const uint32_t slot = index - a;
            if (slot >= tslots) return;          // only reachable with unsorted input
            __hip_atomic_fetch_add(&s_sum[slot], (double)x, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_WORKGROUP);
            __hip_atomic_fetch_or(&s_bits[slot >> 5], 1u << (slot & 31), __ATOMIC_RELAXED,
                                  __HIP_MEMORY_SCOPE_WORKGROUP);
        });
        __syncthreads();
        distinct = bitmap_prefix<WORDS_MAX>(s_bits, s_wprefix, words, s_wave);
        exclusive = place_tile(distinct);
        // a thread writes out the hit slots of one EMIT_BITS-wide piece of a bitmap
        // word: a tile has fewer words than the workgroup has threads, a word up
        // to 32 hits, and the slowest thread sets the pace
        constexpr uint32_t EMIT_BITS = 4, EMIT_PER = 32 / EMIT_BITS;   // bits of a bitmap word per thread
        for (uint32_t u = tid; u < words * EMIT_PER; u += RED_BLOCK) {
            const uint32_t w = u / EMIT_PER, shift = (u % EMIT_PER) * EMIT_BITS;
            const uint32_t word = s_bits[w];
            uint32_t bits = (word >> shift) & ((1u << EMIT_BITS) - 1u);
            uint64_t pos = (uint64_t)exclusive + s_wprefix[w] + (uint32_t)__popc(word & ((1u << shift) - 1u));
            while (bits) {
                const int bit = __ffs(bits) - 1;
                bits &= bits - 1;
                const uint32_t slot = w * 32u + shift + bit;
                if (pos < capacity) {
                    idx_out[pos] = a + slot;
                    val_out[pos] = (float)s_sum[slot];
                }
                ++pos;
            }
        }
        if (dense)
            for (uint32_t s = tid; s < tslots; s += RED_BLOCK) dense[s] = (float)s_sum[s];
    } else if constexpr (CAN_RANK) {
        // ---- sparsely hit region: mark, rank, then sum into accumulator [rank] ----
        for_each_entry(No{}, [&](uint32_t index, float) {
            const uint32_t slot = index - a;
            if (slot < tslots)
                __hip_atomic_fetch_or(&s_bits[slot >> 5], 1u << (slot & 31), __ATOMIC_RELAXED,
                                      __HIP_MEMORY_SCOPE_WORKGROUP);
        });
        __syncthreads();
        distinct = bitmap_prefix<WORDS_MAX>(s_bits, s_wprefix, words, s_wave);
        // the count is known before the sums: publish it now, wait for the others later
        if (tid == 0) scan_publish_early(tile_desc, tile, distinct);
        exclusive = 0;
        const uint32_t rounds = (distinct + C - 1) / C;             // 1, unless the estimate was off
        if (dense) {
            for (uint32_t s = tid; s < tslots; s += RED_BLOCK) dense[s] = 0.0f;
            __syncthreads();                     // zeros land before the values below
        }
        for (uint32_t round = 0; round < rounds; ++round) {
            const uint32_t r0 = round * C;                           // first rank of this round
            if (round) {                                             // the first round starts cleared
                __syncthreads();                                     // previous round fully read
                for (uint32_t s = tid; s < C; s += RED_BLOCK) s_sum[s] = 0.0;
                __syncthreads();
            }
            auto add = [&](uint32_t index, float x) {
                const uint32_t slot = index - a;
                if (slot >= tslots) return;
                const uint32_t below = s_bits[slot >> 5] & ((1u << (slot & 31)) - 1u);
                const uint32_t rank = (uint32_t)s_wprefix[slot >> 5] + (uint32_t)__popc(below) - r0;
                if (rank < C) {
                    __hip_atomic_fetch_add(&s_sum[rank], (double)x, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_WORKGROUP);
                    s_slot[rank] = (uint16_t)slot;       // every hit of the slot writes the same
                }
            };
            for_each_entry(Yes{}, add);
            __syncthreads();
            if (round == 0) exclusive = place_tile(distinct);
            // accumulators and their slots are already in output order
            const uint32_t in_round = distinct - r0 < C ? distinct - r0 : C;
            for (uint32_t k = tid; k < in_round; k += RED_BLOCK) {
                const uint64_t pos = (uint64_t)exclusive + r0 + k;
                const uint32_t slot = s_slot[k];
                const float x = (float)s_sum[k];
                if (pos < capacity) {
                    idx_out[pos] = a + slot;
                    val_out[pos] = x;
                }
                if (dense) dense[slot] = x;
            }
        }
        if (rounds == 0) exclusive = place_tile(0u);   // an empty tile is still a link of the chain
    }
    if (tile == r.ntiles - 1 && tid == 0) {
        const uint64_t total = (uint64_t)exclusive + distinct;
        const bool failed =
            __hip_atomic_load(&hdr->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0;
        nnz[0] = failed ? ~0ull : (total < capacity ? total : capacity);
        nnz[1] = failed ? ~0ull : total;
    }
}

// traffic_only: the measurement entry point okt_stream_gather - the same tiles and
// the same slice table, but the tile kernel is replaced by one that only moves
// the entries (d_nnz_out and d_dense are not used then).
int reduce_launch(const uint32_t* d_idx_cat, const float* d_val_cat,
                  const uint64_t* d_seg_begin, const uint64_t* d_seg_end,
                  uint32_t seg_stride, const uint32_t* d_lo_hi, uint32_t lo,
                  uint32_t hi, uint32_t B, uint32_t P, uint32_t max_width,
                  uint32_t* d_idx_out, float* d_val_out, uint64_t capacity,
                  uint64_t* d_nnz_out, float* d_dense, void* d_ws, size_t ws_bytes,
                  hipStream_t s, bool traffic_only) {
    if (!d_idx_cat || !d_val_cat || !d_seg_begin || !d_seg_end || (!d_nnz_out && !traffic_only))
        return OKT_ERR_INVALID_ARG;
    if (P == 0 || P > 65535 || B == 0 || B > 65535) return OKT_ERR_INVALID_ARG;
    if (capacity > 0 && (!d_idx_out || !d_val_out)) return OKT_ERR_INVALID_ARG;
    if (!aligned(d_idx_cat, 4) || !aligned(d_val_cat, 4) || !aligned(d_seg_begin, 8) || !aligned(d_seg_end, 8) ||
        !aligned(d_nnz_out, 8) || !aligned(d_idx_out, 4) || !aligned(d_val_out, 4) ||
        !aligned(d_dense, 4) || !aligned(d_lo_hi, 4))
        return OKT_ERR_INVALID_ARG;
    // the caller's bound on the size of the union doubles as the density estimate
    ReduceShape shape = reduce_tile_shape(max_width, capacity);
    // The wide dense tile is for throughput.  A launch that cannot fill the chip
    // anyway is nothing but the latency of its tiles: it takes the narrower dense
    // tile of the ranked shape (more, shorter tiles).
    if (shape.kind == RED_DENSE && (uint64_t)B * reduce_tiles(max_width, RED_C) <= 3 * (uint64_t)device_cus())
        shape = ReduceShape{RED_C, RED_RANKED};
    const uint32_t slots = shape.slots;
    const size_t region_bytes = reduce_ws_bytes_region(max_width, P, slots);
    if (region_bytes > 0xffffffffull) return OKT_ERR_INVALID_ARG;
    if (!d_ws || !aligned(d_ws, 256) || ws_bytes < region_bytes * B) return OKT_ERR_WORKSPACE;
    uint64_t tiles = reduce_tiles(max_width, slots);
    if (tiles == 0) tiles = 1;
    const uint32_t table_offset = (uint32_t)(64 + 8 * (tiles + (tiles + 63) / 64));
    const uint64_t cells = (tiles + 1) * P;
    uint64_t sblocks = (cells + 255) / 256;
    if (sblocks > 4096) sblocks = 4096;
    if (cells * B <= 4096) {
        // few cells: a wave each
        hipLaunchKernelGGL(reduce_slices_wave_kernel, dim3((unsigned)((cells + 3) / 4), B),
                           dim3(256), 0, s, d_idx_cat, d_seg_begin, d_seg_end, seg_stride, d_lo_hi,
                           lo, hi, P, max_width, slots, (char*)d_ws, (uint32_t)region_bytes,
                           table_offset, spin_limit_setting());
    } else {
        hipLaunchKernelGGL(reduce_slices_kernel, dim3((unsigned)sblocks, B), dim3(256), 0, s,
                           d_idx_cat, d_seg_begin, d_seg_end, seg_stride, d_lo_hi, lo, hi, P,
                           max_width, slots, (char*)d_ws, (uint32_t)region_bytes, table_offset,
                           spin_limit_setting(), cells * B >= (1u << 17) ? 1u : 0u);
    }
    // entries a contribution is expected to have in a tile: longer slices are read
    // in spans of two or four blocks of 64
    const uint64_t per_slice = capacity / tiles / P;
    const uint32_t span_blocks = per_slice >= 128 ? 4u : per_slice >= 64 ? 2u : 1u;
    if (traffic_only) {
        timing_before(s);
        hipLaunchKernelGGL(gather_ceiling_kernel, dim3((unsigned)tiles, B), dim3(RED_BLOCK), 0, s,
                           d_idx_cat, d_val_cat, d_seg_begin, seg_stride, d_lo_hi, P, max_width, slots,
                           d_idx_out, d_val_out, capacity, (const char*)d_ws, (uint32_t)region_bytes,
                           table_offset);
        timing_after(s);
        return launch_status();
    }
    timing_before(s);
    auto* tile_kernel = shape.kind == RED_SPARSE  ? reduce_tile_kernel<RED_C_SPARSE, RED_S_SPARSE>
                        : shape.kind == RED_DENSE ? reduce_tile_kernel<RED_C_DENSE, RED_C_DENSE>
                                                  : reduce_tile_kernel<RED_C, RED_S_MAX>;
    hipLaunchKernelGGL(tile_kernel, dim3((unsigned)tiles, B), dim3(RED_BLOCK), 0, s,
                       d_idx_cat, d_val_cat, d_seg_begin, seg_stride, d_lo_hi, lo, hi, P, max_width,
                       slots,
                       d_idx_out, d_val_out, capacity, d_nnz_out, d_dense, (char*)d_ws,
                       (uint32_t)region_bytes, table_offset, span_blocks);
    timing_after(s);
    return launch_status();
}

}  // namespace okt

extern "C" int okt_sparse_reduce(const uint32_t* d_idx_cat, const float* d_val_cat,
                                 const uint64_t* d_chunk_off, uint32_t P, uint32_t lo, uint32_t hi,
                                 uint32_t* d_idx_out, float* d_val_out, uint64_t capacity,
                                 uint64_t* d_nnz_out, float* d_dense_out_or_null, void* d_ws,
                                 size_t ws_bytes, void* stream) {
    if (lo > hi) return OKT_ERR_INVALID_ARG;
    if (!d_chunk_off) return OKT_ERR_INVALID_ARG;
    // contribution p = [off[p], off[p+1]): the same vector is the begins and, one on, the ends
    return okt::reduce_launch(d_idx_cat, d_val_cat, d_chunk_off, d_chunk_off + 1, P + 1, nullptr,
                              lo, hi, 1, P, hi - lo,
                              d_idx_out, d_val_out, capacity, d_nnz_out, d_dense_out_or_null,
                              d_ws, ws_bytes, (hipStream_t)stream, false);
}

extern "C" int okt_sparse_reduce_batch(const uint32_t* d_idx_cat, const float* d_val_cat,
                                       const uint64_t* d_chunk_off, const uint32_t* d_lo_hi,
                                       uint32_t B, uint32_t P, uint32_t max_width,
                                       uint32_t* d_idx_out, float* d_val_out, uint64_t capacity,
                                       uint64_t* d_nnz_out, float* d_dense_out_or_null,
                                       void* d_ws, size_t ws_bytes, void* stream) {
    if (!d_lo_hi || !d_chunk_off) return OKT_ERR_INVALID_ARG;
    return okt::reduce_launch(d_idx_cat, d_val_cat, d_chunk_off, d_chunk_off + 1, P + 1, d_lo_hi,
                              0, 0, B, P, max_width,
                              d_idx_out, d_val_out, capacity, d_nnz_out, d_dense_out_or_null,
                              d_ws, ws_bytes, (hipStream_t)stream, false);
}

extern "C" int okt_stream_gather(const uint32_t* d_idx_cat, const float* d_val_cat,
                                 const uint64_t* d_chunk_off, const uint32_t* d_lo_hi, uint32_t B,
                                 uint32_t P, uint32_t max_width, uint32_t* d_idx_out,
                                 float* d_val_out, uint64_t capacity, void* d_ws, size_t ws_bytes,
                                 void* stream) {
    if (!d_lo_hi || !d_chunk_off || !d_idx_out || !d_val_out) return OKT_ERR_INVALID_ARG;
    return okt::reduce_launch(d_idx_cat, d_val_cat, d_chunk_off, d_chunk_off + 1, P + 1, d_lo_hi,
                              0, 0, B, P, max_width, d_idx_out, d_val_out, capacity, nullptr, nullptr,
                              d_ws, ws_bytes, (hipStream_t)stream, true);
}

extern "C" int okt_sparse_reduce_segments(const uint32_t* d_idx_cat, const float* d_val_cat,
                                          const uint64_t* d_seg_begin, const uint64_t* d_seg_end,
                                          uint32_t P, uint32_t lo, uint32_t hi,
                                          uint32_t* d_idx_out, float* d_val_out, uint64_t capacity,
                                          uint64_t* d_nnz_out, float* d_dense_out_or_null,
                                          void* d_ws, size_t ws_bytes, void* stream) {
    if (lo > hi) return OKT_ERR_INVALID_ARG;
    return okt::reduce_launch(d_idx_cat, d_val_cat, d_seg_begin, d_seg_end, P, nullptr, lo, hi, 1, P,
                              hi - lo, d_idx_out, d_val_out, capacity, d_nnz_out,
                              d_dense_out_or_null, d_ws, ws_bytes, (hipStream_t)stream, false);
}
