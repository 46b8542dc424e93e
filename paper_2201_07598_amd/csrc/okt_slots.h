// Threshold select and compaction through per-tile slots: the streaming pass has
// no scan in it (Sec. 3.1.3 threshold selection; Sec. 3.1.2 packaging;
// Algorithm 2, line 6 residual update).
//
// The vector is cut into tiles of SLOT_TILE elements, one per wave.  The first
// pass is a plain streaming kernel of many small workgroups, with no ticket, no
// wait, no barrier, no loop: a wave loads its tile with four 16-byte loads per
// lane, ranks the selected elements with ballots, and writes them into the tile's
// slot (SLOT_C entries of workspace) and their number into counts[tile].  The second
// pass reads the counts only: a chained scan over them gives every tile its
// place in the output.  The third pass, again of many small workgroups, copies
// the entries of the slots there in index order; a tile that selected more than
// its slot holds ("dense") is walked once more, now that its place is known, and
// written directly.  Only the dense tiles are read twice.
#ifndef OKT_SLOTS_H
#define OKT_SLOTS_H

#include "okt_select_kernel.h"
#include "okt_sizes.h"

namespace okt {

struct SlotEntry { uint32_t idx; float val; };
static_assert(sizeof(SlotEntry) == 8, "an entry is one 8-byte store");
static_assert(SLOT_C % 32 == 0 && SLOT_C <= SLOT_TILE, "half a wave copies a slot in whole turns");

constexpr uint32_t SLOT_FEW = 4;                          // entries a lane of the third pass copies by itself
constexpr int SLOT_FILL_BLOCK = 256;                      // 4 waves = 4 tiles per workgroup
static_assert(SLOT_FILL_BLOCK / WAVE == (int)SLOT_GROUP, "a workgroup of the first pass fills one group of slots");
constexpr int SLOT_SCAN_BLOCK = 1024;
static_assert(SLOT_SCAN_BLOCK == (int)SLOT_SCAN_TILES, "one thread per tile and turn");
constexpr int SLOT_EMIT_BLOCK = 256;
constexpr int SLOT_EMIT_TILES = WAVE;                     // tiles per wave of the third pass: one per lane
constexpr int SLOT_FULLER_WORD = 0, SLOT_DENSE_WORD = 1;  // words of the scan header's padding: tiles listed

// Where entry j of a tile's slot lives.  The first SLOT_FEW entries of every slot -
// all there is, as a rule - lie together at the front of the slot area, those of
// the SLOT_GROUP tiles that one workgroup of the first pass fills interleaved in
// one 128-byte line, which the workgroup always writes in full (with zeros where a
// tile has fewer entries).  So the usual stores of the first pass form one more
// dense stream of whole lines, next to the vector's: the L2 hands a whole line to
// memory where a part of a line costs a read-modify-write, a workgroup dirties one
// line instead of four, and consecutive workgroups write consecutive lines.  The
// later entries of the fuller slots follow behind, laid out the same way.
__device__ __forceinline__ uint64_t slot_at(uint64_t tile, uint32_t j, uint32_t ntiles) {
    const uint64_t group = tile / SLOT_GROUP, member = tile % SLOT_GROUP;
    if (j < SLOT_FEW) return group * (SLOT_GROUP * SLOT_FEW) + (uint64_t)j * SLOT_GROUP + member;
    const uint64_t groups = ((uint64_t)ntiles + SLOT_GROUP - 1) / SLOT_GROUP;
    return groups * (SLOT_GROUP * SLOT_FEW) + group * (SLOT_GROUP * (SLOT_C - SLOT_FEW)) +
           (uint64_t)(j - SLOT_FEW) * SLOT_GROUP + member;
}

// The four rounds of a tile, lane l holding base + 256 u + 4 l .. + 3 of round u.
// A tile that runs past the end of the vector is loaded element by element, with
// zeros past the end.
template <bool NT>
__device__ __forceinline__ void tile_load(const float* __restrict__ src, uint64_t base, uint32_t n,
                                          bool whole, float4 (&v)[4]) {
    const int lane = lane_id();
    if (whole) {
        const float4* p = reinterpret_cast<const float4*>(src + base) + lane;
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = load_quad<NT>(p + u * WAVE);
    } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint64_t i = base + 256u * u + 4u * (uint32_t)lane;
            v[u].x = i < n ? src[i] : 0.0f;
            v[u].y = i + 1 < n ? src[i + 1] : 0.0f;
            v[u].z = i + 2 < n ? src[i + 2] : 0.0f;
            v[u].w = i + 3 < n ? src[i + 3] : 0.0f;
        }
    }
}

// Which of the lane's sixteen elements are selected: bit 4u + c for component c
// of round u.  Elements past the end of the vector never are.
template <typename Test>
__device__ __forceinline__ uint32_t tile_test(const float4 (&v)[4], uint64_t base, uint32_t n,
                                              bool whole, Test test) {
    const int lane = lane_id();
    uint32_t bits = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const uint64_t i = base + 256u * u + 4u * (uint32_t)lane;
        if (test(v[u].x) && (whole || i < n)) bits |= 1u << (4 * u);
        if (test(v[u].y) && (whole || i + 1 < n)) bits |= 2u << (4 * u);
        if (test(v[u].z) && (whole || i + 2 < n)) bits |= 4u << (4 * u);
        if (test(v[u].w) && (whole || i + 3 < n)) bits |= 8u << (4 * u);
    }
    return bits;
}

// Feeds the selected elements of a tile to sink(rank, index, value) in index
// order, rank counting from 0; returns their number (wave-uniform).
template <typename Sink>
__device__ __forceinline__ uint32_t tile_rank(const float4 (&v)[4], uint32_t bits, uint64_t base,
                                              Sink&& sink) {
    uint32_t count = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const uint32_t b = bits >> (4 * u);
        count = select_round((uint32_t)base + 256u * u, v[u], (b & 1u) != 0, (b & 2u) != 0,
                             (b & 4u) != 0, (b & 8u) != 0, count, sink);
    }
    return count;
}

// Number of selected elements of the wave's tile (wave-uniform).
__device__ __forceinline__ uint32_t tile_count(uint32_t bits) {
    uint32_t count = 0;
#pragma unroll
    for (int b = 0; b < 16; ++b) count += (uint32_t)__popcll(__ballot((bits >> b) & 1u));
    return count;
}

// The first pass's stores for a tile that selected `count` <= SLOT_C entries.  The
// wave ranks its entries into `stage` (its own SLOT_C entries of LDS) and writes
// them out, zeros up to SLOT_FEW included, with one store instruction per 64
// entries, so that its share of the group's first line goes out at once.  (A
// store per round that selected something, and one more for the zeros, measured
// the same: the pass pays for the lines it dirties, not for store instructions.)
__device__ __forceinline__ void slot_store_tile(SlotEntry* __restrict__ slots, uint64_t tile,
                                                uint32_t count, const float4 (&v)[4], uint32_t bits,
                                                uint64_t base, SlotEntry* stage, uint32_t ntiles) {
    if (count != 0)
        tile_rank(v, bits, base,
                  [&](uint32_t rank, uint32_t i, float x) { stage[rank] = SlotEntry{i, x}; });
    __builtin_amdgcn_wave_barrier();             // the wave's own LDS writes come before its reads
    const uint32_t upto = count > SLOT_FEW ? count : SLOT_FEW;
    for (uint32_t j = (uint32_t)lane_id(); j < upto; j += WAVE)
        slots[slot_at(tile, j, ntiles)] = j < count ? stage[j] : SlotEntry{0u, 0.0f};
}

// The first pass also clears the scan state of the second (header and descriptors,
// `words` 64-bit words; nothing if `state` is null): one launch less, and the
// second pass starts only when the first has ended.
__device__ __forceinline__ void slot_clear_scan_state(uint64_t* __restrict__ state, uint32_t words,
                                                      uint32_t spin_limit) {
    if (blockIdx.x != 0 || state == nullptr) return;
    for (uint32_t i = threadIdx.x; i < words; i += SLOT_FILL_BLOCK)
        state[i] = i == SCAN_SPIN_WORD ? (uint64_t)spin_limit : 0ull;
}

// ---- first pass over a vector that is only read ----
template <bool NT, typename Test>
__device__ __forceinline__ void slot_fill_tile(const float* __restrict__ acc, uint32_t n, Test test,
                                               uint16_t* __restrict__ counts,
                                               SlotEntry* __restrict__ slots, uint32_t tile,
                                               SlotEntry* stage, uint32_t ntiles) {
    const uint64_t base = (uint64_t)tile * SLOT_TILE;
    const bool whole = base + SLOT_TILE <= n;
    float4 v[4];
    tile_load<NT>(acc, base, n, whole, v);
    const uint32_t bits = tile_test(v, base, n, whole, test);
    const uint32_t count = tile_count(bits);
    if (lane_id() == 0) counts[tile] = (uint16_t)count;
    if (count > SLOT_C) return;
    slot_store_tile(slots, tile, count, v, bits, base, stage, ntiles);
}

template <bool NT>
__global__ __launch_bounds__(SLOT_FILL_BLOCK) void slot_fill_kernel(
    const float* __restrict__ acc, uint32_t n, const float* __restrict__ d_threshold,
    uint16_t* __restrict__ counts, SlotEntry* __restrict__ slots, uint32_t ntiles,
    uint64_t* __restrict__ scan_state, uint32_t scan_words, uint32_t spin_limit) {
    __shared__ SlotEntry s_stage[SLOT_FILL_BLOCK / WAVE][SLOT_C];
    slot_clear_scan_state(scan_state, scan_words, spin_limit);
    const uint32_t tile = blockIdx.x * (SLOT_FILL_BLOCK / WAVE) + (threadIdx.x >> 6);
    if (tile >= ntiles) return;
    const float th = *d_threshold;
    SlotEntry* stage = s_stage[threadIdx.x >> 6];
    if (th == th) slot_fill_tile<NT>(acc, n, TestFloat{__builtin_fabsf(th)}, counts, slots, tile, stage, ntiles);
    else slot_fill_tile<NT>(acc, n, TestKey{magnitude_key(th)}, counts, slots, tile, stage, ntiles);
}

// ---- first pass that forms the accumulator on the way ----
// acc = eps + lr * G (product and sum rounded separately) is tested and written
// back as the new residual.  With ZERO set the selected elements of a tile whose
// slot holds them all are written as zeros, so that nothing has to come back to
// them; a dense tile is written as it is and zeroed by the third pass.
template <bool ZERO, bool NT, typename Test>
__device__ __forceinline__ void slot_fill_accumulate_tile(
    const float* __restrict__ grad, float* __restrict__ res, float lr, uint32_t n, Test test,
    uint16_t* __restrict__ counts, SlotEntry* __restrict__ slots, uint32_t tile, SlotEntry* stage,
    uint32_t ntiles) {
    const int lane = lane_id();
    const uint64_t base = (uint64_t)tile * SLOT_TILE;
    const bool whole = base + SLOT_TILE <= n;
    float4 g[4], a[4];
    tile_load<NT>(grad, base, n, whole, g);
    tile_load<NT>(res, base, n, whole, a);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        a[u].x = __fadd_rn(a[u].x, __fmul_rn(lr, g[u].x));
        a[u].y = __fadd_rn(a[u].y, __fmul_rn(lr, g[u].y));
        a[u].z = __fadd_rn(a[u].z, __fmul_rn(lr, g[u].z));
        a[u].w = __fadd_rn(a[u].w, __fmul_rn(lr, g[u].w));
    }
    const uint32_t bits = tile_test(a, base, n, whole, test);
    const uint32_t count = tile_count(bits);
    if (lane == 0) counts[tile] = (uint16_t)count;
    if (count <= SLOT_C) slot_store_tile(slots, tile, count, a, bits, base, stage, ntiles);
    if (ZERO && count <= SLOT_C) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t b = bits >> (4 * u);
            if (b & 1u) a[u].x = 0.0f;
            if (b & 2u) a[u].y = 0.0f;
            if (b & 4u) a[u].z = 0.0f;
            if (b & 8u) a[u].w = 0.0f;
        }
    }
    if (whole) {
        float4* p = reinterpret_cast<float4*>(res + base) + lane;
#pragma unroll
        for (int u = 0; u < 4; ++u) store_quad<NT>(p + u * WAVE, a[u]);
    } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint64_t i = base + 256u * u + 4u * (uint32_t)lane;
            if (i < n) res[i] = a[u].x;
            if (i + 1 < n) res[i + 1] = a[u].y;
            if (i + 2 < n) res[i + 2] = a[u].z;
            if (i + 3 < n) res[i + 3] = a[u].w;
        }
    }
}

template <bool ZERO, bool NT>
__global__ __launch_bounds__(SLOT_FILL_BLOCK) void slot_fill_accumulate_kernel(
    const float* __restrict__ grad, float* __restrict__ res, float lr, uint32_t n,
    const float* __restrict__ d_threshold, uint16_t* __restrict__ counts,
    SlotEntry* __restrict__ slots, uint32_t ntiles, uint64_t* __restrict__ scan_state,
    uint32_t scan_words, uint32_t spin_limit) {
    __shared__ SlotEntry s_stage[SLOT_FILL_BLOCK / WAVE][SLOT_C];
    slot_clear_scan_state(scan_state, scan_words, spin_limit);
    const uint32_t tile = blockIdx.x * (SLOT_FILL_BLOCK / WAVE) + (threadIdx.x >> 6);
    if (tile >= ntiles) return;
    const float th = *d_threshold;
    if (th == th)
        slot_fill_accumulate_tile<ZERO, NT>(grad, res, lr, n, TestFloat{__builtin_fabsf(th)}, counts,
                                            slots, tile, s_stage[threadIdx.x >> 6], ntiles);
    else
        slot_fill_accumulate_tile<ZERO, NT>(grad, res, lr, n, TestKey{magnitude_key(th)}, counts,
                                            slots, tile, s_stage[threadIdx.x >> 6], ntiles);
}

// ---- second pass: the place of every tile ----
// Workgroup `seg` (a ticket) owns 1024 x tpt consecutive tiles, tpt per thread; a
// chained scan over the counts gives place[tile], the number of entries selected
// before the tile.  The workgroup that holds the last tiles writes the totals.
// The tiles that selected more than SLOT_FEW entries are listed on the way, in no
// particular order, for the third pass to share them out evenly: those whose slot
// holds them all from the front of `list`, the dense ones from its back (the list
// has a word per tile, so the two never meet); one atomic per workgroup and kind.
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void slot_scan_kernel(
    const uint16_t* __restrict__ counts, uint32_t* __restrict__ place, uint32_t* __restrict__ list,
    uint32_t ntiles, uint32_t tpt, uint64_t capacity, uint64_t* __restrict__ nnz_out,
    ScanHeader* hdr, uint64_t* seg_desc, uint64_t* group_desc, uint32_t nseg) {
    static_assert(BLOCK == SLOT_SCAN_BLOCK, "one thread per tile and turn");
    constexpr int WAVES = BLOCK / WAVE;
    __shared__ uint32_t s_count[WAVES];
    __shared__ uint32_t s_listed[WAVES];       // fuller tiles in the low half, dense ones in the high half
    __shared__ uint32_t s_seg;
    __shared__ uint32_t s_list_base[2];
    __shared__ uint32_t s_before[2];
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid >> 6;
    if (tid == 0) s_seg = atomicAdd(&hdr->ticket, 1u);
    __syncthreads();
    const uint32_t seg = s_seg;
    const uint64_t first_tile = ((uint64_t)seg * BLOCK + tid) * tpt;
    uint32_t mine = 0, my_listed = 0;
    for (uint32_t k = 0; k < tpt; ++k)
        if (first_tile + k < ntiles) {
            const uint32_t c = counts[first_tile + k];
            mine += c;
            my_listed += c > SLOT_C ? 0x10000u : c > SLOT_FEW ? 1u : 0u;
        }
    // a workgroup has at most 1024 x tpt tiles of either kind; the two sums share a
    // word as long as that stays below 2^16
    const uint32_t inclusive = wave_inclusive_scan(mine);
    const uint32_t listed_inclusive = wave_inclusive_scan(my_listed);
    if (lane == WAVE - 1) {
        s_count[wave] = inclusive;
        s_listed[wave] = listed_inclusive;
    }
    __syncthreads();
    uint32_t aggregate = 0, wave_first = 0, listed_total = 0, listed_first = 0;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
        if (w == wave) {
            wave_first = aggregate;
            listed_first = listed_total;
        }
        aggregate += s_count[w];
        listed_total += s_listed[w];
    }
    const uint32_t group = seg / SCAN_GROUP;
    if (tid == 2 * WAVE && (listed_total & 0xffffu) != 0)
        s_list_base[0] = atomicAdd(&hdr->pad[SLOT_FULLER_WORD], listed_total & 0xffffu);
    if (tid == 3 * WAVE && (listed_total >> 16) != 0)
        s_list_base[1] = atomicAdd(&hdr->pad[SLOT_DENSE_WORD], listed_total >> 16);
    if (wave == 0) {
        const uint32_t before = scan_within_group(hdr, seg_desc, group_desc, seg, aggregate);
        if (lane == 0) s_before[0] = before;
    } else if (wave == 1) {
        const uint32_t before = scan_across_groups(hdr, group_desc, group);
        if (lane == 0) s_before[1] = before;
    }
    __syncthreads();
    const uint32_t exclusive = s_before[0] + s_before[1];
    if (tid == 0 && group != 0 && seg % SCAN_GROUP == SCAN_GROUP - 1)
        scan_close_group(group_desc, group, exclusive + aggregate);

    uint32_t pos = exclusive + wave_first + inclusive - mine;   // below 2^32: at most n entries in all
    const uint32_t listed_before = listed_first + listed_inclusive - my_listed;
    uint32_t fuller_at = (listed_total & 0xffffu) ? s_list_base[0] + (listed_before & 0xffffu) : 0u;
    uint32_t dense_at = (listed_total >> 16) ? s_list_base[1] + (listed_before >> 16) : 0u;
    for (uint32_t k = 0; k < tpt; ++k) {
        const uint64_t t = first_tile + k;
        if (t >= ntiles) break;
        const uint32_t c = counts[t];
        place[t] = pos;
        if (c > SLOT_C) list[ntiles - 1 - dense_at++] = (uint32_t)t;
        else if (c > SLOT_FEW) list[fuller_at++] = (uint32_t)t;
        pos += c;
    }
    if (seg == nseg - 1 && tid == 0) {
        const uint64_t total = (uint64_t)exclusive + aggregate;
        const bool failed =
            __hip_atomic_load(&hdr->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0;
        nnz_out[0] = failed ? ~0ull : (total < capacity ? total : capacity);
        nnz_out[1] = failed ? ~0ull : total;
    }
}

// ---- third pass: the entries go to their places ----
// Three kinds of tile.  Few entries (at most SLOT_FEW, nearly every tile of a
// sparsely selected vector): a wave owns 64 consecutive tiles, one per lane, and a
// lane copies its tile's entries with two loads.  Fuller slots, and dense tiles
// (count above SLOT_C, nothing in the slot): they come in runs, where a layer of
// the model lies above the threshold, so they are taken from the lists of the
// second pass and shared out evenly over all the waves of the launch, wherever
// they lie.  A fuller slot is copied by half a wave, one lane per entry, four
// slots in flight; a dense tile is walked again by a wave, which writes each
// selected element at the tile's place plus its rank.
//
// What still has to happen to the vector where an entry came from: nothing (a
// copy, or candidates), a zero where the entry is written out, or - for the slots
// of a first pass that wrote the zeros itself - the value back where the output
// is full.  Dense tiles were left as they were by every first pass, so
// `DENSE_ZERO` alone says whether the walk zeroes what it writes out.  Entries
// past the end of the output stay in the vector.
enum SlotAfter { SLOT_KEEP = 0, SLOT_ZERO = 1, SLOT_RESTORE = 2 };

template <int AFTER, bool DENSE_ZERO, typename Test>
__device__ __forceinline__ void slot_emit_tiles(float* __restrict__ acc, uint32_t n, Test test,
                                                const uint16_t* __restrict__ counts,
                                                const uint32_t* __restrict__ place,
                                                const SlotEntry* __restrict__ slots,
                                                const uint32_t* __restrict__ list,
                                                const ScanHeader* __restrict__ hdr,
                                                uint32_t ntiles, uint32_t* __restrict__ idx_out,
                                                float* __restrict__ val_out, uint64_t capacity) {
    const int lane = lane_id();
    const uint32_t wave_of_launch = blockIdx.x * (SLOT_EMIT_BLOCK / WAVE) + (threadIdx.x >> 6);
    const uint32_t waves = gridDim.x * (SLOT_EMIT_BLOCK / WAVE);
    auto put = [&](uint64_t pos, uint32_t i, uint32_t bits) {
        if (pos < capacity) {
            idx_out[pos] = i;
            val_out[pos] = __uint_as_float(bits);
            if (AFTER == SLOT_ZERO) acc[i] = 0.0f;
        } else if (AFTER == SLOT_RESTORE) {
            acc[i] = __uint_as_float(bits);
        }
    };
    // The three kinds are independent of one another, and each is a chain of two or
    // three loads that wait for the one before (list -> count and place -> slot or
    // tile).  A wave's first turn at each kind is therefore taken level by level,
    // all kinds at once, so that the chains overlap; what is left after the first
    // turn (long lists only) is taken one kind after the other.
    constexpr uint32_t NONE = 0xffffffffu;
    constexpr int TURNS = SLOT_C / 32;              // entries sub, sub + 32, ... of a fuller slot
    const uint32_t sub = (uint32_t)lane & 31u;
    const uint32_t half_of_launch = 2u * wave_of_launch + ((uint32_t)lane >> 5);
    auto fuller_meta = [&](const uint32_t (&tile)[4], uint32_t (&c)[4], uint32_t (&at)[4]) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            c[u] = 0;
            at[u] = 0;
            if (tile[u] != NONE) {
                c[u] = counts[tile[u]];
                at[u] = place[tile[u]];
            }
        }
    };
    auto fuller_load = [&](const uint32_t (&tile)[4], const uint32_t (&c)[4], SlotEntry (&e)[4][TURNS]) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int v = 0; v < TURNS; ++v)
                if (sub + 32u * v < c[u]) e[u][v] = slots[slot_at(tile[u], sub + 32u * v, ntiles)];
    };
    auto fuller_store = [&](const uint32_t (&c)[4], const uint32_t (&at)[4], const SlotEntry (&e)[4][TURNS]) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int v = 0; v < TURNS; ++v)
                if (sub + 32u * v < c[u])
                    put((uint64_t)at[u] + sub + 32u * v, e[u][v].idx, __float_as_uint(e[u][v].val));
    };
    auto dense_finish = [&](uint64_t tile, uint64_t at, const float4 (&v)[4]) {
        const uint64_t base = tile * SLOT_TILE;
        const uint32_t bits = tile_test(v, base, n, base + SLOT_TILE <= n, test);
        tile_rank(v, bits, base, [&](uint32_t rank, uint32_t i, float x) {
            const uint64_t pos = at + rank;
            if (pos < capacity) {
                idx_out[pos] = i;
                val_out[pos] = x;
                if (DENSE_ZERO) acc[i] = 0.0f;
            }
        });
    };

    // ---- level 1: counts, places and list items (the lists have a word per tile, so
    // an item past a list's end is read, and then dropped, rather than waited for)
    const uint64_t t = (uint64_t)wave_of_launch * WAVE + lane;       // few entries: one lane per tile
    uint32_t few_c = 0;
    uint64_t few_at = 0;
    if (t < ntiles) {                                                // nothing past the last tile
        few_c = counts[t];
        few_at = place[t];
    }
    const uint64_t q0 = 4ull * half_of_launch;                       // fuller slots: half a wave per slot
    uint32_t f_tile[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) f_tile[u] = q0 + u < ntiles ? list[q0 + u] : NONE;
    uint32_t d_tile = wave_of_launch < ntiles ? list[ntiles - 1 - wave_of_launch] : NONE;   // dense: a wave per tile
    const uint32_t nfuller = hdr->pad[SLOT_FULLER_WORD], ndense = hdr->pad[SLOT_DENSE_WORD];
    if (few_c > SLOT_FEW) few_c = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (q0 + u >= nfuller) f_tile[u] = NONE;
    if (wave_of_launch >= ndense) d_tile = NONE;                     // wave-uniform

    // ---- level 2: the few entries, the fuller slots' counts and places, the dense tile
    SlotEntry few_e[SLOT_FEW];
    if (few_c != 0) {
        const SlotEntry* from = slots + slot_at(t, 0, ntiles);
#pragma unroll
        for (uint32_t j = 0; j < SLOT_FEW; ++j) few_e[j] = from[j * SLOT_GROUP];   // padded: all written
    }
    uint32_t f_c[4], f_at[4];
    fuller_meta(f_tile, f_c, f_at);
    float4 d_v[4];
    uint64_t d_at = 0;
    if (d_tile != NONE) {
        d_at = place[d_tile];
        const uint64_t base = (uint64_t)d_tile * SLOT_TILE;
        tile_load<false>(acc, base, n, base + SLOT_TILE <= n, d_v);
    }

    // ---- level 3: the fuller slots' entries; everything else goes out
    SlotEntry f_e[4][TURNS];
    fuller_load(f_tile, f_c, f_e);
#pragma unroll
    for (uint32_t j = 0; j < SLOT_FEW; ++j)
        if (j < few_c) put(few_at + j, few_e[j].idx, __float_as_uint(few_e[j].val));
    if (d_tile != NONE) dense_finish(d_tile, d_at, d_v);
    fuller_store(f_c, f_at, f_e);

    // ---- what long lists leave for further turns
    for (uint64_t q = q0 + 8ull * waves; q < nfuller; q += 8ull * waves) {
#pragma unroll
        for (int u = 0; u < 4; ++u) f_tile[u] = q + u < nfuller ? list[q + u] : NONE;
        fuller_meta(f_tile, f_c, f_at);
        fuller_load(f_tile, f_c, f_e);
        fuller_store(f_c, f_at, f_e);
    }
    for (uint64_t q = (uint64_t)wave_of_launch + waves; q < ndense; q += waves) {
        const uint64_t tile = list[ntiles - 1 - q];
        const uint64_t at = place[tile];
        const uint64_t base = tile * SLOT_TILE;
        tile_load<false>(acc, base, n, base + SLOT_TILE <= n, d_v);
        dense_finish(tile, at, d_v);
    }
}

template <int AFTER, bool DENSE_ZERO>
__global__ __launch_bounds__(SLOT_EMIT_BLOCK) void slot_emit_kernel(
    float* __restrict__ acc, uint32_t n, const float* __restrict__ d_threshold,
    const uint16_t* __restrict__ counts, const uint32_t* __restrict__ place,
    const SlotEntry* __restrict__ slots, const uint32_t* __restrict__ list,
    const ScanHeader* __restrict__ hdr, uint32_t ntiles, uint32_t* __restrict__ idx_out,
    float* __restrict__ val_out, uint64_t capacity) {
    const float th = *d_threshold;
    if (th == th)
        slot_emit_tiles<AFTER, DENSE_ZERO>(acc, n, TestFloat{__builtin_fabsf(th)}, counts, place,
                                           slots, list, hdr, ntiles, idx_out, val_out, capacity);
    else
        slot_emit_tiles<AFTER, DENSE_ZERO>(acc, n, TestKey{magnitude_key(th)}, counts, place, slots,
                                           list, hdr, ntiles, idx_out, val_out, capacity);
}

// ---- host side (okt_select.hip) ----
// Shortest vector that takes the three-pass form, for the plain selects or for the
// calls that form the accumulator on the way (the built-in lengths unless the test
// hook has set another).
uint64_t slot_min_n(bool accumulating);
// Second and third pass of a select through slots; the first pass has filled the
// counts and the slots of the workspace `ws` (laid out by `plan`, scan state
// cleared).  `d_threshold`: what the first pass tested against.  `after`: what the
// entries of the slots still need done to the vector; `dense_zero`: the walk over
// a dense tile zeroes what it writes out.
int launch_slot_finish(float* d_acc, uint64_t n, const float* d_threshold, const SlotPlan& plan,
                       char* ws, int after, bool dense_zero, uint32_t* d_idx_out, float* d_val_out,
                       uint64_t capacity, uint64_t* d_nnz_out, hipStream_t s);

}  // namespace okt
#endif
