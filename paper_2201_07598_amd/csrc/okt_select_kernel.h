// The threshold-select kernel, as a template over its shape.
#ifndef OKT_SELECT_KERNEL_H
#define OKT_SELECT_KERNEL_H

#include <type_traits>

#include "okt_device.h"

namespace okt {

// Lanes below this one that have their bit set in a 64-bit wave mask.
__device__ __forceinline__ uint32_t mask_rank(uint64_t m) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

// How an element is tested against the threshold.  For every threshold that is
// not a NaN, key(x) >= key(th) is the same as !(|x| < |th|) in IEEE arithmetic
// with subnormals kept: one compare with an |.| source modifier per element, a
// NaN x counts as selected just as its key lies above every non-NaN key.  A NaN
// threshold (possible only if the k-th largest magnitude itself is a NaN) takes
// the integer key comparison.
struct TestFloat {
    float th_abs;
    __device__ __forceinline__ bool operator()(float x) const { return !(__builtin_fabsf(x) < th_abs); }
};
struct TestKey {
    uint32_t th_key;
    __device__ __forceinline__ bool operator()(float x) const { return magnitude_key(x) >= th_key; }
};

// A wave's stash in LDS: the selected entries of its piece, in index order, as
// the value (4 bytes) and the position inside the piece (2 bytes: a piece is at
// most SEL_PIECE_MAX = 16,384 elements long).  Six bytes an entry instead of eight
// is a third more entries in the same LDS.
struct StashEntry { uint32_t idx; float val; };
struct WaveStash {
    float* val;
    uint16_t* off;
    uint32_t base;                                   // index of the piece's first element
    __device__ __forceinline__ void put(uint32_t rank, uint32_t i, float x) const {
        val[rank] = x;
        off[rank] = (uint16_t)(i - base);
    }
    __device__ __forceinline__ StashEntry operator[](uint32_t j) const {
        return StashEntry{base + (uint32_t)off[j], val[j]};
    }
};
template <int WAVES, int STASH>
struct StashMemory {                                 // the stashes of a workgroup
    float val[WAVES][STASH];
    uint16_t off[WAVES][STASH];
    __device__ __forceinline__ WaveStash of(int wave, uint64_t piece_start) {
        return WaveStash{val[wave], off[wave], (uint32_t)piece_start};
    }
};

// One round of a wave: 64 lanes x float4 = 256 consecutive elements starting at
// `first` (lane l holds first + 4l .. first + 4l + 3); sx..sw say which of the
// lane's components are selected.  Calls sink(rank, index, value) for every
// selected element, rank counting from `count` in ascending index order, and
// returns the new count (wave-uniform).  Nearly every round that selects
// anything selects at most one component per lane; that case costs one rank
// (a single mbcnt pair) and one sink call.
template <typename Sink>
__device__ __forceinline__ uint32_t select_round(uint32_t first, const float4& v, bool sx, bool sy,
                                                 bool sz, bool sw, uint32_t count, Sink&& sink) {
    const uint64_t bx = __ballot(sx), by = __ballot(sy), bz = __ballot(sz), bw = __ballot(sw);
    const uint64_t bxy = bx | by, bxyz = bxy | bz, any = bxyz | bw;
    if (any == 0) return count;
    const uint32_t i0 = first + 4u * (uint32_t)lane_id();
    const uint64_t multi = (bx & by) | (bxy & bz) | (bxyz & bw);   // lanes selecting 2+ components
    if (multi == 0) {
        if (sx | sy | sz | sw) {
            // exactly one of sx..sw is set.  The components go through an empty
            // asm so that the blend stays three selects; seen as one vector, the
            // compiler turns it into an indexed access through scratch memory.
            float vx = v.x, vy = v.y, vz = v.z, vw = v.w;
            asm volatile("" : "+v"(vx), "+v"(vy), "+v"(vz), "+v"(vw));
            uint32_t comp = 0;
            float x = vx;
            if (sy) { comp = 1; x = vy; }
            if (sz) { comp = 2; x = vz; }
            if (sw) { comp = 3; x = vw; }
            sink(count + mask_rank(any), i0 + comp, x);
        }
        return count + (uint32_t)__popcll(any);
    }
    uint32_t rank = count + mask_rank(bx) + mask_rank(by) + mask_rank(bz) + mask_rank(bw);
    if (sx) sink(rank++, i0, v.x);
    if (sy) sink(rank++, i0 + 1, v.y);
    if (sz) sink(rank++, i0 + 2, v.z);
    if (sw) sink(rank++, i0 + 3, v.w);
    return count + (uint32_t)(__popcll(bx) + __popcll(by) + __popcll(bz) + __popcll(bw));
}

// Where a walk first ran past a limit on its count: the start of that batch of
// rounds and the count there (wave-uniform).  `hit` false: it never did.
struct WalkMark {
    uint64_t at;
    uint32_t count;
    bool hit;
};

// Walks the wave's piece [start, end) of acc in rounds of 256 elements, U rounds
// in flight, and feeds every selected element to `sink` in ascending index
// order, ranks counting from `count`.  Returns the count at the end.  If `mark`
// is given, it records the first batch after which the count exceeds `limit`;
// with STOP the walk ends right there (what it returns is then no total).
template <int U, bool NT = false, bool STOP = false, typename Test, typename Sink>
__device__ __forceinline__ uint32_t select_walk(const float* acc, uint64_t start, uint64_t end,
                                                Test test, Sink&& sink, uint32_t count = 0,
                                                WalkMark* mark = nullptr, uint32_t limit = 0) {
    const int lane = lane_id();
    uint64_t r = start;
    auto note = [&](uint64_t batch_start, uint32_t before) {
        if (mark && !mark->hit && count > limit) *mark = WalkMark{batch_start, before, true};
    };
    float4 v[U], w[U];
    auto load_batch = [&](float4* dst, uint64_t at) {     // start is 16-byte aligned
        const float4* src = reinterpret_cast<const float4*>(acc + at) + lane;
#pragma unroll
        for (int u = 0; u < U; ++u) dst[u] = load_quad<NT>(src + u * WAVE);
    };
    if (r + 256 * U <= end) load_batch(v, r);
    for (; r + 256 * U <= end; r += 256 * U) {
        const uint32_t before = count;
#pragma unroll
        for (int u = 0; u < U; ++u) w[u] = v[u];
        if (r + 2 * 256 * U <= end) load_batch(v, r + 256 * U);
#pragma unroll
        for (int u = 0; u < U; ++u)
            count = select_round((uint32_t)r + 256u * u, w[u], test(w[u].x), test(w[u].y),
                                 test(w[u].z), test(w[u].w), count, sink);
        note(r, before);
        if (STOP && mark->hit) return count;
    }
    for (; r + 256 <= end; r += 256) {                    // whole rounds short of a batch
        const uint32_t before = count;
        const float4 x = load_quad<NT>(reinterpret_cast<const float4*>(acc + r) + lane);
        count = select_round((uint32_t)r, x, test(x.x), test(x.y), test(x.z), test(x.w), count, sink);
        note(r, before);
        if (STOP && mark->hit) return count;
    }
    for (; r < end; r += 256) {                           // the ragged end of the vector
        const uint32_t before = count;
        const uint64_t i = r + 4u * (uint32_t)lane;
        float e[4];
        bool s[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bool inside = i + c < end;
            e[c] = inside ? acc[i + c] : 0.0f;
            s[c] = inside && test(e[c]);
        }
        count = select_round((uint32_t)r, make_float4(e[0], e[1], e[2], e[3]), s[0], s[1], s[2],
                             s[3], count, sink);
        note(r, before);
    }
    return count;
}

// What the select runs over, and what happens to an element of it once its entry
// has been written to the output.  No walk stores into what it reads: a store
// between the loads of a streaming loop makes every later load wait for the
// store's acknowledgement (loads and stores retire through one in-order
// counter), which cost the zeroing select 15 to 40 % of its time.  The zeros are
// written when the entries go out, from the stash, in index order - neighbouring
// lanes, neighbouring addresses - after the walk.
//   stash_emit(walked, i, o)  entry i of the walked array left the stash for
//                             output position holding index o
//   walk_emit(walked, i, o)   the same for an entry written by the second walk of
//                             a piece that overflowed its stash
//   restore                   the first pass already zeroed the stashed entries
//                             (the fused kernel's dense write-back): those that
//                             do not fit the output are put back
// DenseSource: a dense vector whose emitted elements are zeroed (the residual
// update); DenseZeroedSource: the same after a first pass that wrote the zeros of
// the stashed entries itself; DenseCopySource: a dense vector that is only read.
// CooSource: the value array of a sorted COO list, left untouched; the output
// index of position i is idx_in[i].  CandidateSource: a sorted COO list of
// candidates drawn from a dense residual (idx_in set), or that residual itself
// (idx_in null); an entry's place in the residual is zeroed when it goes out.
struct DenseSource {
    static constexpr bool restore = false;
    __device__ __forceinline__ uint32_t out_index(uint32_t i) const { return i; }
    __device__ __forceinline__ void stash_emit(float* walked, uint32_t i, uint32_t) const { walked[i] = 0.0f; }
    __device__ __forceinline__ void walk_emit(float* walked, uint32_t i, uint32_t) const { walked[i] = 0.0f; }
};
struct DenseZeroedSource {
    static constexpr bool restore = true;
    __device__ __forceinline__ uint32_t out_index(uint32_t i) const { return i; }
    __device__ __forceinline__ void stash_emit(float*, uint32_t, uint32_t) const {}
    __device__ __forceinline__ void walk_emit(float* walked, uint32_t i, uint32_t) const { walked[i] = 0.0f; }
};
struct DenseCopySource {
    static constexpr bool restore = false;
    __device__ __forceinline__ uint32_t out_index(uint32_t i) const { return i; }
    __device__ __forceinline__ void stash_emit(float*, uint32_t, uint32_t) const {}
    __device__ __forceinline__ void walk_emit(float*, uint32_t, uint32_t) const {}
};
struct CooSource {
    static constexpr bool restore = false;
    const uint32_t* idx_in;
    __device__ __forceinline__ uint32_t out_index(uint32_t i) const { return idx_in[i]; }
    __device__ __forceinline__ void stash_emit(float*, uint32_t, uint32_t) const {}
    __device__ __forceinline__ void walk_emit(float*, uint32_t, uint32_t) const {}
};
struct CandidateSource {
    static constexpr bool restore = false;
    const uint32_t* idx_in;
    float* res;                              // used only when idx_in is set
    __device__ __forceinline__ uint32_t out_index(uint32_t i) const { return idx_in ? idx_in[i] : i; }
    // `walked` is the array the walk runs over, `i` the position in it, `o` the output index
    __device__ __forceinline__ void stash_emit(float* walked, uint32_t i, uint32_t o) const {
        if (idx_in) res[o] = 0.0f;
        else walked[i] = 0.0f;
    }
    __device__ __forceinline__ void walk_emit(float* walked, uint32_t i, uint32_t o) const {
        stash_emit(walked, i, o);
    }
};

// Second half of a select: the workgroup publishes its count, learns the count of
// everything before it from the chained scan, and each wave writes its pairs to
// their final place.  On entry the wave has seen `count` selected entries in its
// piece [start, end) and holds the first `stashed` of them (in index order) in
// its LDS stash; nothing of the piece has been changed, unless the source says
// that the first pass zeroed the stashed entries itself.  A wave whose stash did
// not hold everything (locally dense selection) writes out the `resume_count`
// entries that lie before `resume_at` and walks the rest of its piece, from
// `resume_at`, a second time, writing directly.
template <int BLOCK, int U, int STASH, bool NT, typename Test, typename Source>
__device__ __forceinline__ void select_finish(
    float* __restrict__ acc, Test test, Source source, uint32_t* __restrict__ idx_out,
    float* __restrict__ val_out, uint64_t capacity, uint64_t* __restrict__ nnz_out,
    ScanHeader* hdr, uint64_t* seg_desc, uint64_t* group_desc, uint32_t nseg, uint32_t seg,
    uint64_t start, uint64_t end, uint32_t count, uint32_t stashed, uint64_t resume_at,
    uint32_t resume_count, WaveStash mine, uint32_t* s_count, uint32_t* s_before) {
    constexpr int WAVES = BLOCK / WAVE;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid >> 6;
    if (lane == 0) s_count[wave] = count;
    __syncthreads();
    uint32_t aggregate = 0, wave_first = 0;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
        if (w == wave) wave_first = aggregate;
        aggregate += s_count[w];
    }

    // ---- position of the segment in the output: two waves, two levels, at once ----
    const uint32_t group = seg / SCAN_GROUP;
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

    // ---- emit in ascending index order ----
    const uint64_t first = (uint64_t)exclusive + wave_first;
    const bool all_stashed = count == stashed;
    const uint32_t final_entries = all_stashed ? count : resume_count;   // of the stash
    for (uint32_t j = lane; j < final_entries; j += WAVE) {
        const uint64_t pos = first + j;
        const StashEntry e = mine[j];
        if (pos < capacity) {
            const uint32_t o = source.out_index(e.idx);
            idx_out[pos] = o;
            val_out[pos] = e.val;
            source.stash_emit(acc, e.idx, o);
        } else if (Source::restore) {
            acc[e.idx] = e.val;             // output full: the entry stays in the residual
        }
    }
    if (!all_stashed) {
        // The rest of the piece, from resume_at on, is walked again, a stash-full at
        // a time: a walk that only reads until the stash has run over, then the
        // entries that lie before the batch in which it did are written out (the
        // positions are known now), and so on from that batch.  Loads and stores
        // stay apart, as in the first walk.  A batch holds at most 256 * U elements,
        // fewer than the stash does, so every turn emits at least one batch.
        static_assert(256 * U <= STASH, "a batch of rounds fits the stash");
        (void)start;
        uint64_t at = resume_at;
        uint32_t done = resume_count;               // entries of the piece written so far
        while (at < end) {
            WalkMark over = {end, 0u, false};
            const uint32_t seen = select_walk<U, NT, true>(
                acc, at, end, test, [&](uint32_t rank, uint32_t i, float x) {
                    if (rank - done < (uint32_t)STASH) mine.put(rank - done, i, x);
                }, done, &over, done + (uint32_t)STASH);
            const uint32_t upto = over.hit ? over.count : seen;
            for (uint32_t j = lane; j < upto - done; j += WAVE) {
                const uint64_t pos = first + done + j;
                const StashEntry e = mine[j];
                if (pos < capacity) {
                    const uint32_t o = source.out_index(e.idx);
                    idx_out[pos] = o;
                    val_out[pos] = e.val;
                    source.walk_emit(acc, e.idx, o);
                }
            }
            if (!over.hit) break;
            at = over.at;
            done = over.count;
        }
    }
    if (seg == nseg - 1 && tid == 0) {
        const uint64_t total = (uint64_t)exclusive + aggregate;
        const bool failed =
            __hip_atomic_load(&hdr->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0;
        nnz_out[0] = failed ? ~0ull : (total < capacity ? total : capacity);
        nnz_out[1] = failed ? ~0ull : total;
    }
}

// Workgroup `seg` (a ticket) owns WAVES consecutive pieces of `piece` elements,
// one per wave.  A wave streams its piece once, with no barrier, no wait and no
// store in the loop, and parks the few selected (index, value) pairs in its LDS
// stash; what the source wants done to an emitted element (the zero of the
// residual update) happens when the stash is written out.
template <int BLOCK, int U, int STASH, bool NT, typename Test, typename Source>
__device__ __forceinline__ void select_body(
    float* __restrict__ acc, uint32_t n, Test test, Source source, uint32_t* __restrict__ idx_out,
    float* __restrict__ val_out, uint64_t capacity, uint64_t* __restrict__ nnz_out,
    ScanHeader* hdr, uint64_t* seg_desc, uint64_t* group_desc, uint32_t nseg, uint32_t piece,
    uint32_t seg, StashMemory<BLOCK / WAVE, STASH>& s_stash, uint32_t* s_count, uint32_t* s_before) {
    constexpr int WAVES = BLOCK / WAVE;
    const int wave = threadIdx.x >> 6;
    const uint64_t start = ((uint64_t)seg * WAVES + wave) * piece;
    const uint64_t end = start + piece < n ? start + piece : n;       // start >= n: empty
    const WaveStash mine = s_stash.of(wave, start);
    WalkMark over = {start, 0u, false};          // the batch in which the stash ran full
    const uint32_t count =
        select_walk<U, NT>(acc, start, end, test, [&](uint32_t rank, uint32_t i, float x) {
            if (rank < (uint32_t)STASH) mine.put(rank, i, x);
        }, 0u, &over, (uint32_t)STASH);
    select_finish<BLOCK, U, STASH, NT>(acc, test, source, idx_out, val_out, capacity, nnz_out, hdr,
                                       seg_desc, group_desc, nseg, seg, start, end, count,
                                       count < (uint32_t)STASH ? count : (uint32_t)STASH, over.at,
                                       over.count, mine, s_count, s_before);
}

// The accumulate and the select in one pass (reuse iterations of Ok-Topk SGD,
// where the threshold is known before the accumulator is): a wave reads its
// piece of the gradient and of the residual, forms acc = eps + lr * G (product
// and sum rounded separately), tests it, parks the selected pairs in its stash
// and writes the new residual -- acc, with zeros at the parked entries -- as
// whole 16-byte stores.  Every residual line is written once, densely: no
// scattered zeroing at all.  Rounds met after the stash is full are written
// unzeroed and left to the second walk of select_finish.  With ZERO false the
// residual is written without the zeros (the parked entries are candidates only:
// the pass that collects them for the exact threshold of a refresh iteration).
template <int BLOCK, int U, int STASH, bool ZERO, bool NT, typename Test>
__device__ __forceinline__ void accumulate_select_body(
    const float* __restrict__ grad, float* __restrict__ res, float lr, uint32_t n, Test test,
    uint32_t* __restrict__ idx_out, float* __restrict__ val_out, uint64_t capacity,
    uint64_t* __restrict__ nnz_out, ScanHeader* hdr, uint64_t* seg_desc, uint64_t* group_desc,
    uint32_t nseg, uint32_t piece, uint32_t seg, StashMemory<BLOCK / WAVE, STASH>& s_stash, uint32_t* s_count,
    uint32_t* s_before) {
    constexpr int WAVES = BLOCK / WAVE;
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x >> 6;
    const uint64_t start = ((uint64_t)seg * WAVES + wave) * piece;
    const uint64_t end = start + piece < n ? start + piece : n;
    const WaveStash mine = s_stash.of(wave, start);
    uint32_t count = 0, stashed = 0;                 // wave-uniform
    uint64_t resume_at = start;                      // first round that was not stashed
    bool resumed = false;

    // one round of 256 elements whose accumulator values are in `a`; returns the
    // residual to store
    auto round = [&](uint32_t first, float4 a, bool sx, bool sy, bool sz, bool sw) -> float4 {
        // the round goes to the stash if all of it fits (and nothing was left out before)
        const uint32_t add = (uint32_t)(__popcll(__ballot(sx)) + __popcll(__ballot(sy)) +
                                        __popcll(__ballot(sz)) + __popcll(__ballot(sw)));
        const bool room = count == stashed && count + add <= (uint32_t)STASH;
        if (!room && !resumed) {
            resumed = true;
            resume_at = first;
        }
        const uint32_t now = select_round(first, a, sx, sy, sz, sw, count,
                                          [&](uint32_t rank, uint32_t i, float x) {
                                              if (room) mine.put(rank, i, x);
                                          });
        if (room) {
            stashed = now;
            if (ZERO) {
                if (sx) a.x = 0.0f;
                if (sy) a.y = 0.0f;
                if (sz) a.z = 0.0f;
                if (sw) a.w = 0.0f;
            }
        }
        count = now;
        return a;
    };
    auto fma2 = [&](float e, float g) { return __fadd_rn(e, __fmul_rn(lr, g)); };

    // The loads of the next batch are issued before the stores of this one: loads
    // and stores retire through one in-order counter, so a load queued behind a
    // store would wait for the store's acknowledgement on every trip.
    uint64_t r = start;
    float4 g[U], e[U];
    auto load_batch = [&](uint64_t at) {
        const float4* gsrc = reinterpret_cast<const float4*>(grad + at) + lane;
        const float4* esrc = reinterpret_cast<const float4*>(res + at) + lane;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            g[u] = load_quad<NT>(gsrc + u * WAVE);
            e[u] = load_quad<NT>(esrc + u * WAVE);
        }
    };
    if (r + 256 * U <= end) load_batch(r);
    for (; r + 256 * U <= end; r += 256 * U) {
        float4 a[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            a[u].x = fma2(e[u].x, g[u].x);
            a[u].y = fma2(e[u].y, g[u].y);
            a[u].z = fma2(e[u].z, g[u].z);
            a[u].w = fma2(e[u].w, g[u].w);
        }
        if (r + 2 * 256 * U <= end) load_batch(r + 256 * U);
        float4* edst = reinterpret_cast<float4*>(res + r) + lane;
#pragma unroll
        for (int u = 0; u < U; ++u)
            store_quad<NT>(edst + u * WAVE, round((uint32_t)r + 256u * u, a[u], test(a[u].x),
                                                  test(a[u].y), test(a[u].z), test(a[u].w)));
    }
    for (; r + 256 <= end; r += 256) {               // whole rounds short of a batch
        const float4 gq = load_quad<NT>(reinterpret_cast<const float4*>(grad + r) + lane);
        const float4 eq = load_quad<NT>(reinterpret_cast<const float4*>(res + r) + lane);
        const float4 a = make_float4(fma2(eq.x, gq.x), fma2(eq.y, gq.y), fma2(eq.z, gq.z),
                                     fma2(eq.w, gq.w));
        reinterpret_cast<float4*>(res + r)[lane] =
            round((uint32_t)r, a, test(a.x), test(a.y), test(a.z), test(a.w));
    }
    for (; r < end; r += 256) {                      // the ragged end of the vector
        const uint64_t i = r + 4u * (uint32_t)lane;
        float a[4];
        bool s[4], inside[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            inside[c] = i + c < end;
            a[c] = inside[c] ? fma2(res[i + c], grad[i + c]) : 0.0f;
            s[c] = inside[c] && test(a[c]);
        }
        const float4 out = round((uint32_t)r, make_float4(a[0], a[1], a[2], a[3]), s[0], s[1],
                                 s[2], s[3]);
        if (inside[0]) res[i] = out.x;
        if (inside[1]) res[i + 1] = out.y;
        if (inside[2]) res[i + 2] = out.z;
        if (inside[3]) res[i + 3] = out.w;
    }
    // every stashed entry lies before resume_at, and is already zeroed where ZERO is set
    using Source = typename std::conditional<ZERO, DenseZeroedSource, DenseCopySource>::type;
    select_finish<BLOCK, U, STASH, NT>(res, test, Source{}, idx_out, val_out, capacity, nnz_out, hdr,
                                       seg_desc, group_desc, nseg, seg, start, end, count, stashed,
                                       resume_at, stashed, mine, s_count, s_before);
}

template <int BLOCK, int U, int STASH, typename Source, bool NT>
__global__ __launch_bounds__(BLOCK) void select_kernel(
    float* __restrict__ acc, uint32_t n, const float* __restrict__ d_threshold,
    uint32_t* __restrict__ idx_out, float* __restrict__ val_out, uint64_t capacity,
    uint64_t* __restrict__ nnz_out, ScanHeader* hdr, uint64_t* seg_desc, uint64_t* group_desc,
    uint32_t nseg, uint32_t piece) {
    static_assert(BLOCK % WAVE == 0 && BLOCK >= 2 * WAVE, "needs two waves for the scan");
    constexpr int WAVES = BLOCK / WAVE;
    __shared__ StashMemory<WAVES, STASH> s_stash;
    __shared__ uint32_t s_count[WAVES];
    __shared__ uint32_t s_seg;
    __shared__ uint32_t s_before[2];           // within the group, across groups

    if (threadIdx.x == 0) s_seg = atomicAdd(&hdr->ticket, 1u);
    __syncthreads();
    const uint32_t seg = s_seg;
    const float th = *d_threshold;
    if (th == th) {
        select_body<BLOCK, U, STASH, NT>(acc, n, TestFloat{__builtin_fabsf(th)}, Source{}, idx_out,
                                             val_out, capacity, nnz_out, hdr, seg_desc,
                                             group_desc, nseg, piece, seg, s_stash, s_count,
                                             s_before);
    } else {
        select_body<BLOCK, U, STASH, NT>(acc, n, TestKey{magnitude_key(th)}, Source{}, idx_out, val_out,
                                             capacity, nnz_out, hdr, seg_desc, group_desc, nseg,
                                             piece, seg, s_stash, s_count, s_before);
    }
}

// The same selection over the values of a sorted COO list whose length is on the
// device (at most max_nnz): entries at or above the threshold are copied, in
// order, with their indices; the input is not modified.
template <int BLOCK, int U, int STASH>
__global__ __launch_bounds__(BLOCK) void coo_select_kernel(
    const uint32_t* __restrict__ idx_in, const float* __restrict__ val_in,
    const uint64_t* __restrict__ d_nnz_in, uint32_t max_nnz,
    const float* __restrict__ d_threshold, uint32_t* __restrict__ idx_out,
    float* __restrict__ val_out, uint64_t capacity, uint64_t* __restrict__ nnz_out,
    ScanHeader* hdr, uint64_t* seg_desc, uint64_t* group_desc, uint32_t nseg, uint32_t piece) {
    constexpr int WAVES = BLOCK / WAVE;
    __shared__ StashMemory<WAVES, STASH> s_stash;
    __shared__ uint32_t s_count[WAVES];
    __shared__ uint32_t s_seg;
    __shared__ uint32_t s_before[2];
    if (threadIdx.x == 0) s_seg = atomicAdd(&hdr->ticket, 1u);
    __syncthreads();
    const uint32_t seg = s_seg;
    const uint64_t have = *d_nnz_in;
    const uint32_t n = have < max_nnz ? (uint32_t)have : max_nnz;
    float* vals = const_cast<float*>(val_in);         // CooSource never writes
    const float th = *d_threshold;
    if (th == th) {
        select_body<BLOCK, U, STASH, false>(vals, n, TestFloat{__builtin_fabsf(th)},
                                             CooSource{idx_in}, idx_out, val_out, capacity,
                                             nnz_out, hdr, seg_desc, group_desc, nseg, piece, seg,
                                             s_stash, s_count, s_before);
    } else {
        select_body<BLOCK, U, STASH, false>(vals, n, TestKey{magnitude_key(th)},
                                             CooSource{idx_in}, idx_out, val_out, capacity,
                                             nnz_out, hdr, seg_desc, group_desc, nseg, piece, seg,
                                             s_stash, s_count, s_before);
    }
}

template <int BLOCK, int U, int STASH, bool NT>
__global__ __launch_bounds__(BLOCK) void accumulate_select_kernel(
    const float* __restrict__ grad, float* __restrict__ res, float lr, uint32_t n,
    const float* __restrict__ d_threshold, uint32_t* __restrict__ idx_out,
    float* __restrict__ val_out, uint64_t capacity, uint64_t* __restrict__ nnz_out,
    ScanHeader* hdr, uint64_t* seg_desc, uint64_t* group_desc, uint32_t nseg, uint32_t piece) {
    constexpr int WAVES = BLOCK / WAVE;
    __shared__ StashMemory<WAVES, STASH> s_stash;
    __shared__ uint32_t s_count[WAVES];
    __shared__ uint32_t s_seg;
    __shared__ uint32_t s_before[2];
    if (threadIdx.x == 0) s_seg = atomicAdd(&hdr->ticket, 1u);
    __syncthreads();
    const uint32_t seg = s_seg;
    const float th = *d_threshold;
    if (th == th) {
        accumulate_select_body<BLOCK, U, STASH, true, NT>(
            grad, res, lr, n, TestFloat{__builtin_fabsf(th)}, idx_out, val_out, capacity, nnz_out,
            hdr, seg_desc, group_desc, nseg, piece, seg, s_stash, s_count, s_before);
    } else {
        accumulate_select_body<BLOCK, U, STASH, true, NT>(
            grad, res, lr, n, TestKey{magnitude_key(th)}, idx_out, val_out, capacity, nnz_out,
            hdr, seg_desc, group_desc, nseg, piece, seg, s_stash, s_count, s_before);
    }
}

}  // namespace okt
#endif
