// okt_topk_threshold_exact: the exact k-th largest |acc| (Algorithm 1, lines
// 2-4, th_re_evaluate; Sec. 3.1.3).  The paper sorts; this is an exact MSD
// radix select over the 31-bit magnitude key, digits of 11 + 11 + 9 bits, most
// significant first (the first digit is the exponent and three mantissa bits).
//
// Per digit: one streaming pass builds a histogram of that digit over the keys
// that match the digits found so far (LDS histogram per workgroup, flushed with
// one global atomic per non-empty bin), then one small workgroup walks the
// histogram from the top to find the bin that holds rank k.  All counts are
// integers, so the result is exact and independent of scheduling.  State lives
// in the workspace on the device; the host never waits.
#include "okt_device.h"
#include "okt_sizes.h"

namespace okt {

struct RadixState {
    uint32_t prefix;       // digits found so far (the high bits of the answer)
    uint32_t pad;
    uint64_t k_rem;        // rank still to find inside the current prefix
    uint64_t above;        // keys strictly above the current prefix
};

constexpr int HIST_BLOCK = 256;
constexpr int HIST_ITERS = 4;                              // float4 per thread per step
constexpr int HIST_STEP4 = HIST_BLOCK * HIST_ITERS;        // float4 per workgroup per step

// One digit pass over the keys.  SHIFT/BITS select the digit; keys take part if
// their bits above the digit equal state->prefix (always, for the first digit).
template <int SHIFT, int BITS, bool FIRST>
__global__ __launch_bounds__(HIST_BLOCK) void radix_hist_kernel(
    const float* __restrict__ acc, uint32_t n, const RadixState* __restrict__ state,
    uint32_t* __restrict__ hist) {
    constexpr int BINS = 1 << BITS;
    __shared__ uint32_t s_hist[BINS];
    for (int b = threadIdx.x; b < BINS; b += HIST_BLOCK) s_hist[b] = 0;
    const uint32_t prefix = FIRST ? 0u : state->prefix;
    __syncthreads();

    auto take = [&](float x) {
        const uint32_t key = magnitude_key(x);
        if (FIRST || (key >> (SHIFT + BITS)) == prefix)
            atomicAdd(&s_hist[(key >> SHIFT) & (BINS - 1)], 1u);
    };

    const uint32_t n4 = n >> 2;
    const float4* src = reinterpret_cast<const float4*>(acc);
    const uint32_t stride = gridDim.x * (uint32_t)HIST_STEP4;
    uint32_t base4 = blockIdx.x * (uint32_t)HIST_STEP4;
    // n4 < 2^30 and stride <= 2^21, so base4 never wraps
    for (; base4 + HIST_STEP4 <= n4; base4 += stride) {
        float4 v[HIST_ITERS];
#pragma unroll
        for (int it = 0; it < HIST_ITERS; ++it) v[it] = src[base4 + it * HIST_BLOCK + threadIdx.x];
#pragma unroll
        for (int it = 0; it < HIST_ITERS; ++it) {
            take(v[it].x); take(v[it].y); take(v[it].z); take(v[it].w);
        }
    }
    // ragged remainder: at most one partial step, owned by the workgroup whose
    // walk lands on it
    if (base4 < n4) {
        for (int it = 0; it < HIST_ITERS; ++it) {
            const uint32_t i = base4 + it * HIST_BLOCK + threadIdx.x;
            if (i < n4) {
                const float4 x = src[i];
                take(x.x); take(x.y); take(x.z); take(x.w);
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 3u)) take(acc[(n4 << 2) + threadIdx.x]);
    __syncthreads();
    for (int b = threadIdx.x; b < BINS; b += HIST_BLOCK) {
        const uint32_t c = s_hist[b];
        if (c) atomicAdd(&hist[b], c);
    }
}

// Walk one histogram from the top bin down to the bin that holds rank k_rem.
template <int BITS, bool LAST>
__global__ __launch_bounds__(256) void radix_pick_kernel(
    RadixState* state, const uint32_t* __restrict__ hist, float* threshold_out,
    uint64_t* count_ge_out) {
    constexpr int BINS = 1 << BITS;
    constexpr int PER = BINS / 256;                  // bins per thread (8 or 2)
    __shared__ uint64_t s_part[256];
    const int t = threadIdx.x;
    // thread t owns bins [BINS - (t+1)*PER, BINS - t*PER): thread 0 the top ones
    uint64_t mine = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) mine += hist[BINS - 1 - (t * PER + j)];
    s_part[t] = mine;
    __syncthreads();
    if (t != 0) return;
    const uint64_t k_rem = state->k_rem;
    uint64_t above = 0;
    int owner = 0;
    while (owner < 255 && above + s_part[owner] < k_rem) above += s_part[owner++];
    int bin = BINS - 1 - owner * PER;
    for (int j = 0; j < PER - 1 && above + hist[bin] < k_rem; ++j) above += hist[bin--];
    // now above < k_rem <= above + hist[bin]
    const uint32_t prefix = (state->prefix << BITS) | (uint32_t)bin;
    state->prefix = prefix;
    state->k_rem = k_rem - above;
    state->above += above;
    if (LAST) {
        *threshold_out = __uint_as_float(prefix);
        *count_ge_out = state->above + hist[bin];
    }
}

__global__ void radix_init_kernel(RadixState* state, uint32_t* hist, uint64_t k) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < 3 * RS_MAX_BINS) hist[i] = 0;
    if (i == 0) {
        state->prefix = 0;
        state->pad = 0;
        state->k_rem = k;
        state->above = 0;
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
    uint32_t* hist1 = (uint32_t*)((char*)d_ws + RS_STATE_BYTES);
    uint32_t* hist2 = hist1 + RS_MAX_BINS;
    uint32_t* hist3 = hist2 + RS_MAX_BINS;

    const uint64_t steps = ((n >> 2) + HIST_STEP4 - 1) / HIST_STEP4;
    unsigned grid = (unsigned)(steps < 2048 ? (steps ? steps : 1) : 2048);

    hipLaunchKernelGGL(radix_init_kernel, dim3(3 * RS_MAX_BINS / 256), dim3(256), 0, s, state,
                       hist1, k);
    hipLaunchKernelGGL((radix_hist_kernel<20, RS_BITS1, true>), dim3(grid), dim3(HIST_BLOCK), 0, s,
                       d_acc, (uint32_t)n, state, hist1);
    hipLaunchKernelGGL((radix_pick_kernel<RS_BITS1, false>), dim3(1), dim3(256), 0, s, state,
                       hist1, d_threshold_out, d_count_ge_out);
    hipLaunchKernelGGL((radix_hist_kernel<9, RS_BITS2, false>), dim3(grid), dim3(HIST_BLOCK), 0, s,
                       d_acc, (uint32_t)n, state, hist2);
    hipLaunchKernelGGL((radix_pick_kernel<RS_BITS2, false>), dim3(1), dim3(256), 0, s, state,
                       hist2, d_threshold_out, d_count_ge_out);
    hipLaunchKernelGGL((radix_hist_kernel<0, RS_BITS3, false>), dim3(grid), dim3(HIST_BLOCK), 0, s,
                       d_acc, (uint32_t)n, state, hist3);
    hipLaunchKernelGGL((radix_pick_kernel<RS_BITS3, true>), dim3(1), dim3(256), 0, s, state,
                       hist3, d_threshold_out, d_count_ge_out);
    return hipGetLastError() == hipSuccess ? OKT_OK : OKT_ERR_HIP;
}
