// okt_topk_threshold_exact: the exact k-th largest |acc| (Algorithm 1, lines
// 2-4, th_re_evaluate; Sec. 3.1.3).  The paper sorts; this is an exact
// selection on the 31-bit magnitude key that reads the vector about once.
//
//   1. A histogram of the first digit (exponent and three mantissa bits) over a
//      strided sample of about a million elements gives a key that lies, with a
//      wide margin, below the k-th largest one.
//   2. One streaming pass over the whole vector copies every key at or above
//      that bound, a little more than k of them, to the workspace (the select
//      kernel's loop: one compare per element, per-wave LDS stash, one global
//      atomic per workgroup for what the stashes hold at the end).
//   3. If at least k keys were collected (always, unless the sample misled),
//      rank k is among them, and an exact MSD radix select, digits of
//      11 + 11 + 9 bits, runs over the candidates only.  Otherwise, or when the
//      vector is short or the workspace small, the same radix select runs over
//      the whole vector (three more passes).
// Six launches at most: wherever a complete histogram has to be read, the
// workgroup that added its counts last does the reading, in the same launch.
// Either way the answer is the exact order statistic: all arithmetic is integer
// counting, the sample only decides how much is read.  State lives in the
// workspace on the device; the host never waits.
//
// okt_accumulate_topk_select: a whole refresh iteration (Algorithm 2, lines 4-6,
// with the threshold re-evaluated) that reads the gradient and the residual
// once.  The sample is formed on the fly from both; the pass that collects the
// candidates is the fused accumulate+select kernel run against the sample's
// bound, writing the accumulator over the residual and the candidates, in index
// order with their indices, to the workspace; the radix select runs over the
// candidate values; and the final select walks the candidates instead of the
// vector, zeroing the residual where an entry goes out.  If the sample misled,
// the last two steps run over the whole vector instead: same results.
#include "okt_device.h"
#include "okt_select_kernel.h"
#include "okt_sizes.h"
#include "okt_slots.h"

namespace okt {

struct RadixState {
    uint32_t prefix;       // digits found so far (the high bits of the answer)
    uint32_t use_cand;     // 1: the radix passes run over the candidate keys
    uint64_t k_rem;        // rank still to find inside the current prefix
    uint64_t above;        // keys strictly above the current prefix
    uint64_t m;            // number of 32-bit words the radix passes run over
    uint32_t cand_lo;      // every key >= cand_lo is a candidate
    uint32_t pad;
    unsigned long long cand_count;    // number of candidates found by the counting pass
    uint32_t done[4];      // workgroups that have handed in their histogram: sample, digits 1-3
    uint64_t collected[2]; // ordered collection (refresh iteration): candidates written, found
};
static_assert(sizeof(RadixState) <= RS_STATE_BYTES, "state fits its slot");

constexpr int HIST_BLOCK = 256;
constexpr int HIST_ITERS = 4;                              // float4 per thread per step
constexpr int HIST_STEP4 = HIST_BLOCK * HIST_ITERS;        // float4 per workgroup per step

// Find the bin that holds rank k_rem counting from the top bin down: 256 threads,
// thread t owns the PER bins below the (t * PER) highest ones; an inclusive scan
// over the threads' sums names the owner, who walks its own few bins.  The
// owner (exactly one thread) stores (bin, keys above the bin) to s_result.
template <int BITS>
__device__ __forceinline__ void pick_bin(const uint32_t* __restrict__ hist, uint64_t k_rem,
                                         uint64_t* s_wave_total, uint64_t* s_result) {
    constexpr int BINS = 1 << BITS;
    constexpr int PER = BINS / 256;                  // bins per thread (8 or 2)
    const int t = threadIdx.x, lane = t & (WAVE - 1), wave = t >> 6;
    uint32_t c[PER];
    uint64_t mine = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        // j = 0 is the thread's highest bin; the counts were added by other workgroups
        c[j] = __hip_atomic_load(&hist[BINS - 1 - (t * PER + j)], __ATOMIC_RELAXED,
                                 __HIP_MEMORY_SCOPE_AGENT);
        mine += c[j];
    }
    const uint64_t incl = wave_inclusive_scan<uint64_t>(mine);
    if (lane == WAVE - 1) s_wave_total[wave] = incl;
    __syncthreads();
    uint64_t before = incl - mine;
    for (int w = 0; w < wave; ++w) before += s_wave_total[w];
    if (before < k_rem && k_rem <= before + mine) {  // true for exactly one thread
        uint64_t above = before;
        int j = 0;
        while (j < PER - 1 && above + c[j] < k_rem) above += c[j++];
        s_result[0] = (uint64_t)(BINS - 1 - (t * PER + j));
        s_result[1] = above;                         // above < k_rem <= above + hist[bin]
    }
    __syncthreads();
}

// Adds a workgroup's counts to the global histogram and waits for the answers: an
// atomic that has returned has been carried out where every CU sees it, which a
// release fence would only achieve by writing the whole L2 back.
template <int BINS>
__device__ __forceinline__ void add_counts(uint32_t* __restrict__ hist, const uint32_t* s_hist) {
    uint32_t seen = 0;
#pragma unroll
    for (int b = threadIdx.x; b < BINS; b += HIST_BLOCK) {     // all out first, then one wait
        const uint32_t c = s_hist[b];
        if (c) seen |= atomicAdd(&hist[b], c);
    }
    asm volatile("" ::"v"(seen));
}
// True in exactly one workgroup of the grid: the one that comes last.  Called by
// every workgroup once add_counts has returned; the last one may then
// read the complete histogram (with device-scope loads).
__device__ __forceinline__ bool last_workgroup(uint32_t* counter, uint32_t* s_flag) {
    __syncthreads();
    if (threadIdx.x == 0) *s_flag = atomicAdd(counter, 1u) == gridDim.x - 1 ? 1u : 0u;
    __syncthreads();
    return *s_flag != 0;
}

// ---------------------------------------------------------------------------
// radix passes (over the candidates, or over the whole vector)
// ---------------------------------------------------------------------------
// One digit pass.  SHIFT/BITS select the digit; a key takes part if its bits
// above the digit equal state->prefix (always, for the first digit).  The source
// is the candidate array or the vector itself, as the state says; both are
// arrays of 32-bit words whose low 31 bits are the key.
// The first pass also decides what the passes run over: the candidates, if the
// counting pass ran and rank k is among them, else the whole vector.  The
// workgroup that hands in its counts last picks the digit (the bin that holds
// the rank still sought) and leaves the state for the next pass; after the last
// digit it writes the threshold and its count.
template <int SHIFT, int BITS, int PASS>
__global__ __launch_bounds__(HIST_BLOCK) void radix_hist_kernel(
    const float* __restrict__ acc, const uint32_t* __restrict__ cand, RadixState* state,
    uint32_t* __restrict__ hist, uint64_t n, uint64_t k, uint64_t cand_cap, int sampled,
    float* threshold_out, uint64_t* count_ge_out) {
    constexpr int BINS = 1 << BITS;
    constexpr bool FIRST = PASS == 1, LAST = PASS == 3;
    static_assert(HIST_BLOCK == 256, "pick_bin is written for 256 threads");
    __shared__ uint32_t s_hist[BINS];
    __shared__ uint64_t s_wave_total[4], s_result[2];
    __shared__ uint32_t s_flag;
    uint32_t use_cand;
    uint64_t m64;
    if (FIRST) {
        // keys at or above cand_lo: counted by the collect pass, or by the ordered
        // collection of a refresh iteration (all ones if one of its waits gave up)
        const uint64_t found = sampled == 2 ? state->collected[1] : state->cand_count;
        use_cand = sampled && k <= found && found <= cand_cap ? 1u : 0u;   // rank k is among them
        m64 = use_cand ? found : n;
    } else {
        use_cand = state->use_cand;
        m64 = state->m;
    }
    const uint32_t* src = use_cand ? cand : reinterpret_cast<const uint32_t*>(acc);
    const uint32_t m = (uint32_t)m64;
    const uint32_t m4 = m >> 2;
    uint32_t base4 = blockIdx.x * (uint32_t)HIST_STEP4;
    for (int b = threadIdx.x; b < BINS; b += HIST_BLOCK) s_hist[b] = 0;
    const uint32_t prefix = FIRST ? 0u : state->prefix;
    const uint64_t k_rem = FIRST ? k : state->k_rem;
    const uint64_t above_so_far = FIRST ? 0ull : state->above;
    __syncthreads();

    auto take = [&](uint32_t word) {
        const uint32_t key = word & ABS_MASK;
        if (FIRST || (key >> (SHIFT + BITS)) == prefix)
            atomicAdd(&s_hist[(key >> SHIFT) & (BINS - 1)], 1u);
    };
    const uint4* src4 = reinterpret_cast<const uint4*>(src);
    const uint32_t stride = gridDim.x * (uint32_t)HIST_STEP4;
    // m4 < 2^30 and stride <= 2^21, so base4 never wraps
    // a pass over the whole of a vector longer than the last-level cache finds nothing
    // of it there (wave-uniform choice)
    const bool around_cache = !use_cand && m64 >= STREAM_PAST_CACHE_N;
    for (; base4 + HIST_STEP4 <= m4; base4 += stride) {
        uint4 v[HIST_ITERS];
#pragma unroll
        for (int it = 0; it < HIST_ITERS; ++it) {
            const uint4* at = src4 + base4 + it * HIST_BLOCK + threadIdx.x;
            if (around_cache) {
                typedef uint32_t v4u __attribute__((ext_vector_type(4)));
                const v4u q = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(at));
                v[it] = make_uint4(q.x, q.y, q.z, q.w);
            } else {
                v[it] = *at;
            }
        }
#pragma unroll
        for (int it = 0; it < HIST_ITERS; ++it) {
            take(v[it].x); take(v[it].y); take(v[it].z); take(v[it].w);
        }
    }
    if (base4 < m4) {       // ragged remainder: one partial step, owned by one workgroup
        for (int it = 0; it < HIST_ITERS; ++it) {
            const uint32_t i = base4 + it * HIST_BLOCK + threadIdx.x;
            if (i < m4) {
                const uint4 x = src4[i];
                take(x.x); take(x.y); take(x.z); take(x.w);
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (m & 3u)) take(src[(m4 << 2) + threadIdx.x]);
    __syncthreads();
    add_counts<BINS>(hist, s_hist);
    if (!last_workgroup(&state->done[PASS], &s_flag)) return;

    // ---- the complete histogram: pick the digit ----
    pick_bin<BITS>(hist, k_rem, s_wave_total, s_result);
    if (threadIdx.x != 0) return;
    const int bin = (int)s_result[0];
    const uint64_t above = s_result[1];
    const uint32_t found = (prefix << BITS) | (uint32_t)bin;
    state->prefix = found;
    state->k_rem = k_rem - above;
    state->above = above_so_far + above;
    if (FIRST) {
        state->use_cand = use_cand;
        state->m = m64;
    }
    if (LAST) {
        *threshold_out = __uint_as_float(found);
        *count_ge_out = above_so_far + above +
                        __hip_atomic_load(&hist[bin], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ---------------------------------------------------------------------------
// sampling, candidate range, counting pass
// ---------------------------------------------------------------------------
// First-digit histogram over every `stride`-th block of 1024 elements.  A
// workgroup takes SAMPLE_PER_WG sampled blocks with all their loads in flight,
// so that few workgroups (few global atomics per hot bin) still cover the
// sample at memory latency.  The workgroup that comes last reads the bound off
// the complete histogram: the first-digit bin that holds the sample rank
// k' + margin, k' = k * sample / n; every key from the bottom of that bin up is
// a candidate.
constexpr int SAMPLE_PER_WG = 8;
// With `grad` set the sampled values are eps + lr * G formed on the fly (`acc` is
// then the residual before the accumulate).
__global__ __launch_bounds__(HIST_BLOCK) void sample_hist_kernel(
    const float* __restrict__ acc, const float* __restrict__ grad, float lr,
    uint32_t nblocks_sampled, uint32_t stride, uint32_t* __restrict__ hist, RadixState* state,
    uint64_t n, uint64_t k) {
    constexpr int BINS = 1 << RS_BITS1;
    __shared__ uint32_t s_hist[BINS];
    __shared__ uint64_t s_wave_total[4], s_result[2];
    __shared__ uint32_t s_flag;
    for (int b = threadIdx.x; b < BINS; b += HIST_BLOCK) s_hist[b] = 0;
    __syncthreads();
    // sampled blocks are whole: the host only samples the first floor(n/1024) blocks
    float4 v[SAMPLE_PER_WG];
#pragma unroll
    for (int u = 0; u < SAMPLE_PER_WG; ++u) {
        const uint32_t j = blockIdx.x * SAMPLE_PER_WG + u;
        v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (j < nblocks_sampled) {
            const size_t at = (size_t)j * stride * 256 + threadIdx.x;
            v[u] = reinterpret_cast<const float4*>(acc)[at];
            if (grad) {
                const float4 g = reinterpret_cast<const float4*>(grad)[at];
                v[u].x = __fadd_rn(v[u].x, __fmul_rn(lr, g.x));
                v[u].y = __fadd_rn(v[u].y, __fmul_rn(lr, g.y));
                v[u].z = __fadd_rn(v[u].z, __fmul_rn(lr, g.z));
                v[u].w = __fadd_rn(v[u].w, __fmul_rn(lr, g.w));
            }
        }
    }
#pragma unroll
    for (int u = 0; u < SAMPLE_PER_WG; ++u) {
        if (blockIdx.x * SAMPLE_PER_WG + u < nblocks_sampled) {
            atomicAdd(&s_hist[magnitude_key(v[u].x) >> 20], 1u);
            atomicAdd(&s_hist[magnitude_key(v[u].y) >> 20], 1u);
            atomicAdd(&s_hist[magnitude_key(v[u].z) >> 20], 1u);
            atomicAdd(&s_hist[magnitude_key(v[u].w) >> 20], 1u);
        }
    }
    __syncthreads();
    add_counts<BINS>(hist, s_hist);
    if (!last_workgroup(&state->done[0], &s_flag)) return;

    const uint64_t sample = (uint64_t)nblocks_sampled * 1024;
    // k' rounded up; margin of 16 standard deviations of a binomial count, and some
    const uint64_t kp = (k * sample + n - 1) / n;      // k, sample < 2^32: no overflow
    uint64_t margin = 64;
    while (margin * margin < 256 * kp) margin += margin / 2 + 1;     // ~ 16 sqrt(k')
    uint64_t r_lo = kp + margin;                                     // a sample rank safely below the target
    if (r_lo > sample) r_lo = sample;
    pick_bin<RS_BITS1>(hist, r_lo, s_wave_total, s_result);
    if (threadIdx.x == 0) state->cand_lo = (uint32_t)s_result[0] << 20;
}

constexpr int CNT_BLOCK = SEL_BLOCK;
constexpr int CNT_WAVES = CNT_BLOCK / WAVE;
constexpr int CNT_STASH = 1024;                  // keys per wave between flushes
constexpr int CNT_U = 4;

// The counting pass: one contiguous piece per wave, as in the select kernel,
// with the same one-compare-per-element test.  Every key at or above cand_lo is
// a candidate and is copied to `cand`, in any order (per-wave LDS stash; a stash
// that fills up is flushed with an atomic of its own, the rest of a workgroup
// with one atomic at the end).
template <bool NT, typename Test>
__device__ __forceinline__ void collect_body(const float* __restrict__ acc, uint32_t n,
                                             uint32_t piece, RadixState* state,
                                             uint32_t* __restrict__ cand, uint64_t cand_cap,
                                             Test test, uint32_t (*s_stash)[CNT_STASH],
                                             uint32_t* s_left, unsigned long long* s_base) {
    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane(tid >> 6);
    const uint64_t start = ((uint64_t)blockIdx.x * CNT_WAVES + wave) * piece;
    const uint64_t end = start + piece < n ? start + piece : n;
    uint32_t* mine = s_stash[wave];
    uint32_t stashed = 0;                        // wave-uniform

    auto flush = [&]() {
        if (stashed == 0) return;
        unsigned long long base = 0;
        if (lane == 0) base = atomicAdd(&state->cand_count, (unsigned long long)stashed);
        base = __shfl(base, 0, WAVE);
        for (uint32_t j = lane; j < stashed; j += WAVE)
            if (base + j < cand_cap) cand[base + j] = mine[j];
        stashed = 0;
    };
    auto round = [&](const float4& v, bool cx, bool cy, bool cz, bool cw) {
        if (stashed > (uint32_t)(CNT_STASH - 256)) flush();     // room for a whole round
        stashed = select_round(0u, v, cx, cy, cz, cw, stashed,
                               [&](uint32_t rank, uint32_t, float x) { mine[rank] = magnitude_key(x); });
    };

    uint64_t r = start;
    for (; r + 256 * CNT_U <= end; r += 256 * CNT_U) {
        const float4* src = reinterpret_cast<const float4*>(acc + r) + lane;
        float4 v[CNT_U];
#pragma unroll
        for (int u = 0; u < CNT_U; ++u) v[u] = load_quad<NT>(src + u * WAVE);
#pragma unroll
        for (int u = 0; u < CNT_U; ++u)
            round(v[u], test(v[u].x), test(v[u].y), test(v[u].z), test(v[u].w));
    }
    for (; r + 256 <= end; r += 256) {                    // whole rounds short of a batch
        const float4 v = load_quad<NT>(reinterpret_cast<const float4*>(acc + r) + lane);
        round(v, test(v.x), test(v.y), test(v.z), test(v.w));
    }
    for (; r < end; r += 256) {                           // the ragged end of the vector
        const uint64_t i = r + 4u * (uint32_t)lane;
        float e[4];
        bool c[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool inside = i + j < end;
            e[j] = inside ? acc[i + j] : 0.0f;
            c[j] = inside && test(e[j]);
        }
        round(make_float4(e[0], e[1], e[2], e[3]), c[0], c[1], c[2], c[3]);
    }
    // What is left goes out with ONE atomic per workgroup: atomics on a single
    // address retire one after the other, and one per wave (tens of thousands on a
    // long vector) would outlast the whole pass.
    if (lane == 0) s_left[wave] = stashed;
    __syncthreads();
    if (tid == 0) {
        uint32_t total = 0;
#pragma unroll
        for (int w = 0; w < CNT_WAVES; ++w) total += s_left[w];
        *s_base = total ? atomicAdd(&state->cand_count, (unsigned long long)total) : 0ull;
    }
    __syncthreads();
    unsigned long long base = *s_base;
    for (uint32_t w = 0; w < wave; ++w) base += s_left[w];
    for (uint32_t j = lane; j < stashed; j += WAVE)
        if (base + j < cand_cap) cand[base + j] = mine[j];
}

template <bool NT>
__global__ __launch_bounds__(CNT_BLOCK) void collect_kernel(
    const float* __restrict__ acc, uint32_t n, uint32_t piece, RadixState* state,
    uint32_t* __restrict__ cand, uint64_t cand_cap) {
    __shared__ uint32_t s_stash[CNT_WAVES][CNT_STASH];
    __shared__ uint32_t s_left[CNT_WAVES];
    __shared__ unsigned long long s_base;
    const float lo = __uint_as_float(state->cand_lo);       // a key below the Inf/NaN range, or NaN
    if (lo == lo)
        collect_body<NT>(acc, n, piece, state, cand, cand_cap, TestFloat{lo}, s_stash, s_left, &s_base);
    else
        collect_body<NT>(acc, n, piece, state, cand, cand_cap, TestKey{state->cand_lo}, s_stash, s_left,
                         &s_base);
}

__global__ void radix_init_kernel(RadixState* state, uint32_t* hist, uint32_t words) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < words) hist[i] = 0;
    if (i == 0) {
        RadixState z = {};
        *state = z;
    }
}

// ---------------------------------------------------------------------------
// refresh iteration in one pass over the gradient
// ---------------------------------------------------------------------------
// Clears the radix state, the histograms and the two scan states (collection,
// final select) of a refresh iteration.
__global__ void refresh_init_kernel(RadixState* state, uint32_t* hist, uint32_t hist_words,
                                    uint64_t* scan_a, uint32_t words_a, uint64_t* scan_b,
                                    uint32_t words_b, uint32_t spin_limit) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < hist_words) hist[i] = 0;
    const uint64_t w = i == SCAN_SPIN_WORD ? (uint64_t)spin_limit : 0ull;
    if (i < words_a) scan_a[i] = w;
    if (i < words_b) scan_b[i] = w;
    if (i == 0) {
        RadixState z = {};
        *state = z;
    }
}

// The fused accumulate+select kernel run against the sample's bound: the
// residual becomes the accumulator (no zeros), every element at or above the
// bound goes, in index order, to the candidate list, whose length (written,
// found) lands in state->collected.
template <int BLOCK, int U, int STASH, bool NT>
__global__ __launch_bounds__(BLOCK) void accumulate_collect_kernel(
    const float* __restrict__ grad, float* __restrict__ res, float lr, uint32_t n, RadixState* state,
    uint32_t* __restrict__ cand_idx, float* __restrict__ cand_val, uint64_t cand_cap,
    ScanHeader* hdr, uint64_t* seg_desc, uint64_t* group_desc, uint32_t nseg, uint32_t piece) {
    constexpr int WAVES = BLOCK / WAVE;
    __shared__ StashMemory<WAVES, STASH> s_stash;
    __shared__ uint32_t s_count[WAVES];
    __shared__ uint32_t s_seg;
    __shared__ uint32_t s_before[2];
    if (threadIdx.x == 0) s_seg = atomicAdd(&hdr->ticket, 1u);
    __syncthreads();
    const uint32_t seg = s_seg;
    const uint32_t lo_key = state->cand_lo;
    const float lo = __uint_as_float(lo_key);               // a key below the Inf/NaN range, or NaN
    if (lo == lo) {
        accumulate_select_body<BLOCK, U, STASH, false, NT>(
            grad, res, lr, n, TestFloat{lo}, cand_idx, cand_val, cand_cap, state->collected, hdr,
            seg_desc, group_desc, nseg, piece, seg, s_stash, s_count, s_before);
    } else {
        accumulate_select_body<BLOCK, U, STASH, false, NT>(
            grad, res, lr, n, TestKey{lo_key}, cand_idx, cand_val, cand_cap, state->collected, hdr,
            seg_desc, group_desc, nseg, piece, seg, s_stash, s_count, s_before);
    }
}

// The select of a refresh iteration.  If the radix passes ran over the
// candidates, so does this: the candidates hold every element at or above the
// threshold, in index order, so the walk over them emits what a walk over the
// vector would, and the residual is zeroed where an entry is written out.  The
// candidates are shared out over all the workgroups of the launch.  Otherwise
// the walk runs over the residual itself.
template <int BLOCK, int U, int STASH>
__global__ __launch_bounds__(BLOCK) void candidate_select_kernel(
    float* __restrict__ res, uint32_t n, const RadixState* __restrict__ state,
    const uint32_t* __restrict__ cand_idx, float* __restrict__ cand_val,
    const float* __restrict__ d_threshold, uint32_t* __restrict__ idx_out,
    float* __restrict__ val_out, uint64_t capacity, uint64_t* __restrict__ nnz_out,
    ScanHeader* hdr, uint64_t* seg_desc, uint64_t* group_desc, uint32_t nseg, uint32_t piece) {
    constexpr int WAVES = BLOCK / WAVE;
    __shared__ StashMemory<WAVES, STASH> s_stash;
    __shared__ uint32_t s_count[WAVES];
    __shared__ uint32_t s_seg;
    __shared__ uint32_t s_before[2];
    const bool use_cand = state->use_cand != 0;
    float* walked = res;
    uint32_t len = n;
    CandidateSource source{nullptr, res};
    if (use_cand) {
        walked = cand_val;
        len = (uint32_t)state->m;                           // candidates found: at most n
        source.idx_in = cand_idx;
        const uint32_t waves = nseg * (uint32_t)WAVES;
        uint32_t share = ((len + waves - 1) / waves + 255u) / 256u * 256u;   // whole rounds
        if (share == 0) share = 256u;
        if (share < piece) piece = share;                   // never longer than the launch's piece
        // The launch is sized for a walk over the whole residual; the candidates
        // fill only the first few segments.  The workgroups beyond them leave before
        // they take a ticket (tickets on one counter are served one after the other,
        // some 30 ns each: over a thousand idle workgroups queuing for theirs took
        // longer than the selection itself), so the tickets 0 .. used - 1 go to the
        // `used` workgroups that stay, all of them running.
        const uint32_t per_seg = piece * (uint32_t)WAVES;
        uint32_t used = (len + per_seg - 1) / per_seg;
        if (used == 0) used = 1;
        if (used < nseg) nseg = used;
        if (blockIdx.x >= nseg) return;
    }
    if (threadIdx.x == 0) s_seg = atomicAdd(&hdr->ticket, 1u);
    __syncthreads();
    const uint32_t seg = s_seg;
    const float th = *d_threshold;
    if (th == th) {
        select_body<BLOCK, U, STASH, false>(walked, len, TestFloat{__builtin_fabsf(th)}, source, idx_out,
                                           val_out, capacity, nnz_out, hdr, seg_desc, group_desc,
                                           nseg, piece, seg, s_stash, s_count, s_before);
    } else {
        select_body<BLOCK, U, STASH, false>(walked, len, TestKey{magnitude_key(th)}, source, idx_out,
                                           val_out, capacity, nnz_out, hdr, seg_desc, group_desc,
                                           nseg, piece, seg, s_stash, s_count, s_before);
    }
}

}  // namespace okt

extern "C" int okt_topk_threshold_exact(const float* d_acc, uint64_t n, uint64_t k,
                                        float* d_threshold_out, uint64_t* d_count_ge_out,
                                        void* d_ws, size_t ws_bytes, void* stream) {
    using namespace okt;
    hipStream_t s = (hipStream_t)stream;
    if (!d_acc || !d_threshold_out || !d_count_ge_out) return OKT_ERR_INVALID_ARG;
    if (n == 0 || n > 0xffffffffull || k == 0 || k > n) return OKT_ERR_INVALID_ARG;
    if (!aligned(d_acc, 16) || !aligned(d_threshold_out, 4) || !aligned(d_count_ge_out, 8))
        return OKT_ERR_INVALID_ARG;
    if (!d_ws || !aligned(d_ws, 256) || ws_bytes < threshold_ws_min_bytes())
        return OKT_ERR_WORKSPACE;
    RadixState* state = (RadixState*)d_ws;
    uint32_t* hist_sample = (uint32_t*)((char*)d_ws + RS_STATE_BYTES);
    uint32_t* hist1 = hist_sample + RS_MAX_BINS;
    uint32_t* hist2 = hist1 + RS_MAX_BINS;
    uint32_t* hist3 = hist2 + RS_MAX_BINS;
    uint32_t* cand = hist3 + RS_MAX_BINS;
    const uint64_t cand_cap = (ws_bytes - threshold_ws_min_bytes()) / 4;

    hipLaunchKernelGGL(radix_init_kernel, dim3(4 * RS_MAX_BINS / 256), dim3(256), 0, s, state,
                       hist_sample, 4u * RS_MAX_BINS);

    // sampling pays once the vector is long and the workspace can hold the candidates
    const uint64_t blocks = n / 1024;                       // whole blocks of 1024 elements
    const bool sampled = n >= RS_SAMPLE_MIN_N && cand_cap >= n / 16;
    if (sampled) {
        uint64_t stride = blocks / RS_SAMPLE_BLOCKS;
        if (stride < 1) stride = 1;
        const uint64_t nsamp = (blocks + stride - 1) / stride;
        hipLaunchKernelGGL(sample_hist_kernel,
                           dim3((unsigned)((nsamp + SAMPLE_PER_WG - 1) / SAMPLE_PER_WG)),
                           dim3(HIST_BLOCK), 0, s, d_acc, (const float*)nullptr, 0.0f,
                           (uint32_t)nsamp, (uint32_t)stride, hist_sample, state, n, k);
        static_assert(CNT_WAVES == SEL_WAVES, "the collect pass is cut like the select");
        const SelectShape shape = select_shape(n, device_cus());
        timing_before(s);
        hipLaunchKernelGGL(stream_past_cache(n) ? collect_kernel<true> : collect_kernel<false>,
                           dim3(shape.nseg), dim3(CNT_BLOCK), 0, s, d_acc, (uint32_t)n, shape.piece,
                           state, cand, cand_cap);
        timing_after(s);
    }

    // the radix passes are sized for the candidates when sampling ran (a failed
    // check makes them walk the whole vector with the same, smaller grid)
    const uint64_t expect = sampled ? n / 16 : n;
    const uint64_t steps = ((expect >> 2) + HIST_STEP4 - 1) / HIST_STEP4;
    // every workgroup ends with up to 2048 returning atomics on the shared histogram:
    // over the candidates (a few MB) a workgroup per CU is plenty, over a whole
    // vector the passes want the memory parallelism of many more
    const uint64_t grid_max = sampled ? device_cus() : 8 * device_cus();
    const unsigned grid = (unsigned)(steps < grid_max ? (steps ? steps : 1) : grid_max);
    const int was_sampled = sampled ? 1 : 0;
    hipLaunchKernelGGL((radix_hist_kernel<20, RS_BITS1, 1>), dim3(grid), dim3(HIST_BLOCK), 0, s,
                       d_acc, cand, state, hist1, n, k, cand_cap, was_sampled, d_threshold_out,
                       d_count_ge_out);
    hipLaunchKernelGGL((radix_hist_kernel<9, RS_BITS2, 2>), dim3(grid), dim3(HIST_BLOCK), 0, s,
                       d_acc, cand, state, hist2, n, k, cand_cap, was_sampled, d_threshold_out,
                       d_count_ge_out);
    hipLaunchKernelGGL((radix_hist_kernel<0, RS_BITS3, 3>), dim3(grid), dim3(HIST_BLOCK), 0, s,
                       d_acc, cand, state, hist3, n, k, cand_cap, was_sampled, d_threshold_out,
                       d_count_ge_out);
    return launch_status();
}

extern "C" int okt_accumulate_topk_select(const float* d_grad, float* d_residual_inout, float lr,
                                          uint64_t n, uint64_t k, float* d_threshold_out,
                                          uint64_t* d_count_ge_out, uint32_t* d_idx_out,
                                          float* d_val_out, uint64_t capacity, uint64_t* d_nnz_out,
                                          void* d_ws, size_t ws_bytes, void* stream) {
    using namespace okt;
    hipStream_t s = (hipStream_t)stream;
    if (!d_grad || !d_residual_inout || d_grad == d_residual_inout || !d_threshold_out ||
        !d_count_ge_out || !d_nnz_out)
        return OKT_ERR_INVALID_ARG;
    if (n == 0 || n > 0xffffffffull || k == 0 || k > n) return OKT_ERR_INVALID_ARG;
    if (!aligned(d_grad, 16) || !aligned(d_residual_inout, 16) || !aligned(d_threshold_out, 4) ||
        !aligned(d_count_ge_out, 8) || !aligned(d_nnz_out, 8))
        return OKT_ERR_INVALID_ARG;
    if (capacity > 0 && (!d_idx_out || !d_val_out || !aligned(d_idx_out, 4) ||
                         !aligned(d_val_out, 4)))
        return OKT_ERR_INVALID_ARG;
    const size_t separate = threshold_ws_min_bytes() > select_ws_bytes(n) ? threshold_ws_min_bytes()
                                                                           : select_ws_bytes(n);
    if (!d_ws || !aligned(d_ws, 256) || ws_bytes < separate) return OKT_ERR_WORKSPACE;

    const SelectShape shape = select_shape(n, device_cus());
    const size_t scan_bytes = refresh_scan_bytes(n);
    // The collection of the candidates goes through per-tile slots where the vector
    // is long enough and the workspace has room for them next to the candidates;
    // else through the chained scan of the one-kernel select.
    const SlotPlan plan = slot_plan(n, device_cus());
    const size_t slot_bytes = round_up_256(plan.bytes);
    bool slots = n >= slot_min_n(true) && ws_bytes > threshold_ws_min_bytes() + scan_bytes + slot_bytes;
    size_t fixed = threshold_ws_min_bytes() + scan_bytes + (slots ? slot_bytes : scan_bytes);
    uint64_t cand_cap = ws_bytes > fixed ? ((ws_bytes - fixed) / 8) & ~(uint64_t)63 : 0;
    if (slots && cand_cap < n / 16) {
        slots = false;
        fixed = threshold_ws_min_bytes() + 2 * scan_bytes;
        cand_cap = ws_bytes > fixed ? ((ws_bytes - fixed) / 8) & ~(uint64_t)63 : 0;
    }
    if (n < RS_SAMPLE_MIN_N || cand_cap < n / 16) {
        // short vector (or a workspace without room for candidates): the three steps
        // one after the other, each with the workspace to itself
        int rc = okt_residual_accumulate(d_grad, d_residual_inout, lr, n, stream);
        if (rc != OKT_OK) return rc;
        rc = okt_topk_threshold_exact(d_residual_inout, n, k, d_threshold_out, d_count_ge_out, d_ws,
                                      ws_bytes, stream);
        if (rc != OKT_OK) return rc;
        return okt_threshold_select(d_residual_inout, n, d_threshold_out, d_idx_out, d_val_out,
                                    capacity, d_nnz_out, d_ws, ws_bytes, stream);
    }

    RadixState* state = (RadixState*)d_ws;
    uint32_t* hist_sample = (uint32_t*)((char*)d_ws + RS_STATE_BYTES);
    uint32_t* hist1 = hist_sample + RS_MAX_BINS;
    uint32_t* hist2 = hist1 + RS_MAX_BINS;
    uint32_t* hist3 = hist2 + RS_MAX_BINS;
    char* scan_b = (char*)d_ws + threshold_ws_min_bytes();          // the final select's
    char* scan_a = scan_b + scan_bytes;                             // the collection's, or the slots
    float* cand_val = (float*)(scan_a + (slots ? slot_bytes : scan_bytes));
    uint32_t* cand_idx = (uint32_t*)(cand_val + cand_cap);
    auto header = [](char* p) { return (ScanHeader*)p; };
    auto segs = [](char* p) { return (uint64_t*)(p + SCAN_HEADER_BYTES); };

    const uint32_t words_b = (uint32_t)(scan_ws_bytes(shape.nseg) / 8);
    const uint32_t words_a = slots ? (uint32_t)(scan_ws_bytes(plan.nseg) / 8) : words_b;
    uint32_t init_words = 4u * RS_MAX_BINS;
    if (words_a > init_words) init_words = words_a;
    if (words_b > init_words) init_words = words_b;
    hipLaunchKernelGGL(refresh_init_kernel, dim3((init_words + 255) / 256), dim3(256), 0, s, state,
                       hist_sample, 4u * RS_MAX_BINS, (uint64_t*)scan_a, words_a, (uint64_t*)scan_b,
                       words_b, spin_limit_setting());

    const uint64_t blocks = n / 1024;
    uint64_t stride = blocks / RS_SAMPLE_BLOCKS;
    if (stride < 1) stride = 1;
    const uint64_t nsamp = (blocks + stride - 1) / stride;
    hipLaunchKernelGGL(sample_hist_kernel,
                       dim3((unsigned)((nsamp + SAMPLE_PER_WG - 1) / SAMPLE_PER_WG)),
                       dim3(HIST_BLOCK), 0, s, d_residual_inout, d_grad, lr, (uint32_t)nsamp,
                       (uint32_t)stride, hist_sample, state, n, k);
    if (slots) {
        // the sample's bound is a magnitude key, so its bits read as an fp32 are the
        // bound itself: the slot kernels take it for their threshold
        const float* bound = reinterpret_cast<const float*>(&state->cand_lo);
        timing_before(s);
        auto* fill = stream_past_cache(n) ? slot_fill_accumulate_kernel<false, true>
                                          : slot_fill_accumulate_kernel<false, false>;
        constexpr uint32_t per_wg = SLOT_FILL_BLOCK / WAVE;
        hipLaunchKernelGGL(fill, dim3((plan.ntiles + per_wg - 1) / per_wg), dim3(SLOT_FILL_BLOCK), 0,
                           s, d_grad, d_residual_inout, lr, (uint32_t)n, bound,
                           (uint16_t*)(scan_a + plan.counts_at), (SlotEntry*)(scan_a + plan.slots_at),
                           plan.ntiles, (uint64_t*)nullptr, 0u, 0u);      // refresh_init_kernel cleared it
        timing_after(s);
        const int rc = launch_slot_finish(d_residual_inout, n, bound, plan, scan_a, SLOT_KEEP, false,
                                          cand_idx, cand_val, cand_cap, state->collected, s);
        if (rc != OKT_OK) return rc;
    } else {
        timing_before(s);
        auto* collect = stream_past_cache(n)
                            ? accumulate_collect_kernel<SEL_BLOCK, SEL_U, SEL_STASH, true>
                            : accumulate_collect_kernel<SEL_BLOCK, SEL_U, SEL_STASH, false>;
        hipLaunchKernelGGL(collect, dim3(shape.nseg), dim3(SEL_BLOCK), 0, s, d_grad, d_residual_inout,
                           lr, (uint32_t)n, state, cand_idx, cand_val, cand_cap, header(scan_a),
                           segs(scan_a), segs(scan_a) + shape.nseg, shape.nseg, shape.piece);
        timing_after(s);
    }

    const uint64_t steps = (((n / 16) >> 2) + HIST_STEP4 - 1) / HIST_STEP4;
    const uint64_t one_per_cu = device_cus();
    const unsigned grid = (unsigned)(steps < one_per_cu ? (steps ? steps : 1) : one_per_cu);
    const uint32_t* cand_keys = reinterpret_cast<const uint32_t*>(cand_val);
    hipLaunchKernelGGL((radix_hist_kernel<20, RS_BITS1, 1>), dim3(grid), dim3(HIST_BLOCK), 0, s,
                       d_residual_inout, cand_keys, state, hist1, n, k, cand_cap, 2, d_threshold_out,
                       d_count_ge_out);
    hipLaunchKernelGGL((radix_hist_kernel<9, RS_BITS2, 2>), dim3(grid), dim3(HIST_BLOCK), 0, s,
                       d_residual_inout, cand_keys, state, hist2, n, k, cand_cap, 2, d_threshold_out,
                       d_count_ge_out);
    hipLaunchKernelGGL((radix_hist_kernel<0, RS_BITS3, 3>), dim3(grid), dim3(HIST_BLOCK), 0, s,
                       d_residual_inout, cand_keys, state, hist3, n, k, cand_cap, 2, d_threshold_out,
                       d_count_ge_out);
    hipLaunchKernelGGL((candidate_select_kernel<SEL_BLOCK, SEL_U, SEL_STASH>), dim3(shape.nseg),
                       dim3(SEL_BLOCK), 0, s, d_residual_inout, (uint32_t)n, state, cand_idx, cand_val,
                       d_threshold_out, d_idx_out, d_val_out, capacity, d_nnz_out, header(scan_b),
                       segs(scan_b), segs(scan_b) + shape.nseg, shape.nseg, shape.piece);
    return launch_status();
}
