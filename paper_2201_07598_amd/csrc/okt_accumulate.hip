// okt_residual_accumulate: acc = eps + lr * G  (Algorithm 2, line 4).
//
// HBM-bound streaming kernel: 8 B read + 4 B written per element.  Each thread
// keeps ACC_ITERS 16-byte loads of both inputs in flight before the first use;
// a wave reads 1 KiB contiguous per load instruction; vectors far longer than the
// last-level cache are read and written with the non-temporal hint.  The product and the sum
// are rounded separately (no fused multiply-add), so the result is the same as
// two fp32 tensor operations.
#include "okt_device.h"
#include "okt_sizes.h"

namespace okt {

constexpr int ACC_BLOCK = 256;
constexpr int ACC_ITERS = 4;
constexpr int ACC_TILE4 = ACC_BLOCK * ACC_ITERS;     // float4 per workgroup

__device__ __forceinline__ float acc_one(float e, float g, float lr) {
    return __fadd_rn(e, __fmul_rn(lr, g));
}

template <bool NT>
__global__ __launch_bounds__(ACC_BLOCK) void accumulate_kernel(
    const float* __restrict__ grad, float* __restrict__ res, float lr, uint32_t n) {
    const uint32_t n4 = n >> 2;
    const uint32_t base4 = blockIdx.x * (uint32_t)ACC_TILE4;
    const float4* g4 = reinterpret_cast<const float4*>(grad);
    float4* e4 = reinterpret_cast<float4*>(res);
    float4 g[ACC_ITERS], e[ACC_ITERS];
    if (base4 + ACC_TILE4 <= n4) {
#pragma unroll
        for (int it = 0; it < ACC_ITERS; ++it) {
            const uint32_t i = base4 + it * ACC_BLOCK + threadIdx.x;
            g[it] = load_quad<NT>(g4 + i);
            e[it] = load_quad<NT>(e4 + i);
        }
#pragma unroll
        for (int it = 0; it < ACC_ITERS; ++it) {
            const uint32_t i = base4 + it * ACC_BLOCK + threadIdx.x;
            float4 r;
            r.x = acc_one(e[it].x, g[it].x, lr);
            r.y = acc_one(e[it].y, g[it].y, lr);
            r.z = acc_one(e[it].z, g[it].z, lr);
            r.w = acc_one(e[it].w, g[it].w, lr);
            store_quad<NT>(e4 + i, r);
        }
        return;
    }
    // ragged last workgroup: whole float4 first, then the n % 4 scalars
    for (int it = 0; it < ACC_ITERS; ++it) {
        const uint32_t i = base4 + it * ACC_BLOCK + threadIdx.x;
        if (i < n4) {
            const float4 gg = g4[i];
            float4 r = e4[i];
            r.x = acc_one(r.x, gg.x, lr);
            r.y = acc_one(r.y, gg.y, lr);
            r.z = acc_one(r.z, gg.z, lr);
            r.w = acc_one(r.w, gg.w, lr);
            e4[i] = r;
        }
    }
    const uint32_t tail = (n4 << 2) + threadIdx.x;
    if (threadIdx.x < 4 && tail < n) res[tail] = acc_one(res[tail], grad[tail], lr);
}

}  // namespace okt

extern "C" int okt_residual_accumulate(const float* d_grad, float* d_residual_inout, float lr,
                                       uint64_t n, void* stream) {
    using namespace okt;
    if (n == 0) return OKT_OK;
    if (!d_grad || !d_residual_inout || n > 0xffffffffull) return OKT_ERR_INVALID_ARG;
    if (!aligned(d_grad, 16) || !aligned(d_residual_inout, 16)) return OKT_ERR_INVALID_ARG;
    const uint64_t n4 = n >> 2;
    // the last workgroup also owns the n % 4 scalars, so there is always one
    const uint64_t blocks = n4 / ACC_TILE4 + 1;
    timing_before((hipStream_t)stream);
    auto* kernel = stream_past_cache(n) ? accumulate_kernel<true> : accumulate_kernel<false>;
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(ACC_BLOCK), 0, (hipStream_t)stream,
                       d_grad, d_residual_inout, lr, (uint32_t)n);
    timing_after((hipStream_t)stream);
    return launch_status();
}
