// A host program that uses the library the way a C or C++ caller would: device
// memory from hipMalloc, the default stream, no Python and no torch.  One small
// pass of the hot path (accumulate, exact threshold, select, partition, reduce)
// whose expected results follow from the definitions by plain host code: the
// k-th largest magnitude by std::nth_element, the selection by a filter, the
// quantile boundaries by indexing, and a reduce of the selection with itself
// (every value doubled, exactly); then the first three calls again as the one
// call okt_accumulate_topk_select, which must give the same bits.  Prints
// "cabi smoke ok" and exits 0, or says what differs and exits 1.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "okt.h"

#define HIP_OK(call)                                                                      \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess) {                                                           \
            std::printf("%s failed: %s\n", #call, hipGetErrorString(e_));                 \
            return 1;                                                                     \
        }                                                                                 \
    } while (0)
#define OKT_OK_(call)                                                                     \
    do {                                                                                  \
        int s_ = (call);                                                                  \
        if (s_ != OKT_OK) {                                                               \
            std::printf("%s failed: %s (%s)\n", #call, okt_status_string(s_),             \
                        okt_last_hip_error());                                            \
            return 1;                                                                     \
        }                                                                                 \
    } while (0)

static uint32_t key(float x) {
    uint32_t b;
    std::memcpy(&b, &x, 4);
    return b & 0x7fffffffu;
}

template <typename T>
static int upload(T** d, const std::vector<T>& h) {
    HIP_OK(hipMalloc((void**)d, std::max<size_t>(h.size(), 1) * sizeof(T)));
    HIP_OK(hipMemcpy(*d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice));
    return 0;
}

int main() {
    const uint64_t n = 4500003, k = 20000;     // long enough for the one-pass refresh iteration
    const uint32_t R = 4;
    std::vector<float> g(n), zero(n, 0.0f);
    uint32_t state = 12345u;
    for (uint64_t i = 0; i < n; ++i) {                    // a fixed pseudo-random pattern in (-0.5, 0.5)
        state = state * 1664525u + 1013904223u;
        g[i] = (float)(state >> 8) / 16777216.0f - 0.5f;
    }
    float *d_g = nullptr, *d_res = nullptr, *d_th = nullptr, *d_val = nullptr, *d_oval = nullptr;
    uint32_t *d_idx = nullptr, *d_bounds = nullptr, *d_oidx = nullptr, *d_cat_i = nullptr;
    float* d_cat_v = nullptr;
    uint64_t *d_cnt = nullptr, *d_nnz = nullptr, *d_off = nullptr, *d_chunk = nullptr, *d_onnz = nullptr;
    void* d_ws = nullptr;
    const uint64_t cap = 4 * k;
    if (upload(&d_g, g) || upload(&d_res, zero)) return 1;
    HIP_OK(hipMalloc((void**)&d_th, 4));
    HIP_OK(hipMalloc((void**)&d_cnt, 8));
    HIP_OK(hipMalloc((void**)&d_idx, cap * 4));
    HIP_OK(hipMalloc((void**)&d_val, cap * 4));
    HIP_OK(hipMalloc((void**)&d_nnz, 16));
    HIP_OK(hipMalloc((void**)&d_bounds, (R + 1) * 4));
    HIP_OK(hipMalloc((void**)&d_off, (R + 1) * 8));
    const size_t ws_bytes = okt_workspace_bytes(n, 2);
    HIP_OK(hipMalloc(&d_ws, ws_bytes));
    HIP_OK(hipMemset(d_ws, 0xA5, ws_bytes));              // the library must not rely on a clean workspace

    OKT_OK_(okt_residual_accumulate(d_g, d_res, 1.0f, n, nullptr));
    OKT_OK_(okt_topk_threshold_exact(d_res, n, k, d_th, d_cnt, d_ws, ws_bytes, nullptr));
    OKT_OK_(okt_threshold_select(d_res, n, d_th, d_idx, d_val, cap, d_nnz, d_ws, ws_bytes, nullptr));
    OKT_OK_(okt_region_partition(d_idx, d_nnz, n, R, d_bounds, d_off, nullptr));
    HIP_OK(hipDeviceSynchronize());

    // ---- what the definitions say ----
    std::vector<uint32_t> keys(n);
    for (uint64_t i = 0; i < n; ++i) keys[i] = key(g[i]);          // acc = 0 + 1.0 * g = g, bit for bit
    std::vector<uint32_t> sorted(keys);
    std::nth_element(sorted.begin(), sorted.begin() + (n - k), sorted.end());
    const uint32_t th_key = sorted[n - k];
    std::vector<uint32_t> want_idx;
    std::vector<float> want_val;
    for (uint64_t i = 0; i < n; ++i)
        if (keys[i] >= th_key) {
            want_idx.push_back((uint32_t)i);
            want_val.push_back(g[i]);
        }
    float th;
    uint64_t cnt, nnz[2];
    HIP_OK(hipMemcpy(&th, d_th, 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(&cnt, d_cnt, 8, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(nnz, d_nnz, 16, hipMemcpyDeviceToHost));
    if (key(th) != th_key || th < 0.0f || cnt != want_idx.size()) {
        std::printf("threshold differs: %a / %llu, expected key %08x / %zu\n", th,
                    (unsigned long long)cnt, th_key, want_idx.size());
        return 1;
    }
    if (nnz[0] != want_idx.size() || nnz[1] != want_idx.size()) {
        std::printf("select count differs\n");
        return 1;
    }
    std::vector<uint32_t> idx(nnz[0]);
    std::vector<float> val(nnz[0]), res(n);
    HIP_OK(hipMemcpy(idx.data(), d_idx, nnz[0] * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(val.data(), d_val, nnz[0] * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(res.data(), d_res, n * 4, hipMemcpyDeviceToHost));
    if (idx != want_idx || std::memcmp(val.data(), want_val.data(), val.size() * 4) != 0) {
        std::printf("selected entries differ\n");
        return 1;
    }
    for (uint64_t i = 0, j = 0; i < n; ++i) {
        const bool taken = j < idx.size() && idx[j] == i;
        const float expect = taken ? 0.0f : g[i];
        if (taken) ++j;
        if (std::memcmp(&res[i], &expect, 4) != 0) {
            std::printf("residual differs at %llu\n", (unsigned long long)i);
            return 1;
        }
    }
    std::vector<uint32_t> bounds(R + 1);
    std::vector<uint64_t> off(R + 1);
    HIP_OK(hipMemcpy(bounds.data(), d_bounds, (R + 1) * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(off.data(), d_off, (R + 1) * 8, hipMemcpyDeviceToHost));
    for (uint32_t r = 0; r <= R; ++r) {
        const uint32_t b = r == 0 ? 0u : r == R ? (uint32_t)n : idx[(uint64_t)r * idx.size() / R];
        const uint64_t o = std::lower_bound(idx.begin(), idx.end(), b) - idx.begin();
        if (bounds[r] != b || off[r] != (r == R ? idx.size() : o)) {
            std::printf("partition differs at boundary %u\n", r);
            return 1;
        }
    }

    // ---- the selection reduced with itself over region 1: every value doubled ----
    const uint32_t lo = bounds[1], hi = bounds[2];
    std::vector<uint32_t> cat_i(idx);
    cat_i.insert(cat_i.end(), idx.begin(), idx.end());
    std::vector<float> cat_v(val);
    cat_v.insert(cat_v.end(), val.begin(), val.end());
    std::vector<uint64_t> chunk = {0, idx.size(), 2 * idx.size()};
    if (upload(&d_cat_i, cat_i) || upload(&d_cat_v, cat_v) || upload(&d_chunk, chunk)) return 1;
    HIP_OK(hipMalloc((void**)&d_oidx, cat_i.size() * 4));
    HIP_OK(hipMalloc((void**)&d_oval, cat_i.size() * 4));
    HIP_OK(hipMalloc((void**)&d_onnz, 16));
    OKT_OK_(okt_sparse_reduce(d_cat_i, d_cat_v, d_chunk, 2, lo, hi, d_oidx, d_oval, cat_i.size(),
                              d_onnz, nullptr, d_ws, ws_bytes, nullptr));
    HIP_OK(hipDeviceSynchronize());
    uint64_t onnz[2];
    HIP_OK(hipMemcpy(onnz, d_onnz, 16, hipMemcpyDeviceToHost));
    const uint64_t first = off[1], count = off[2] - off[1];
    if (onnz[0] != count || onnz[1] != count) {
        std::printf("reduce count differs: %llu, expected %llu\n", (unsigned long long)onnz[1],
                    (unsigned long long)count);
        return 1;
    }
    std::vector<uint32_t> oidx(count);
    std::vector<float> oval(count);
    HIP_OK(hipMemcpy(oidx.data(), d_oidx, count * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(oval.data(), d_oval, count * 4, hipMemcpyDeviceToHost));
    for (uint64_t j = 0; j < count; ++j) {
        const float expect = 2.0f * val[first + j];                 // exact in fp32
        if (oidx[j] != idx[first + j] || std::memcmp(&oval[j], &expect, 4) != 0) {
            std::printf("reduce differs at %llu\n", (unsigned long long)j);
            return 1;
        }
    }
    // ---- the iteration again in one call: the same threshold, selection and residual ----
    uint32_t* d_idx2 = nullptr;
    float* d_val2 = nullptr;
    HIP_OK(hipMalloc((void**)&d_idx2, cap * 4));
    HIP_OK(hipMalloc((void**)&d_val2, cap * 4));
    HIP_OK(hipMemset(d_res, 0, n * 4));
    HIP_OK(hipMemset(d_ws, 0x5A, ws_bytes));
    OKT_OK_(okt_accumulate_topk_select(d_g, d_res, 1.0f, n, k, d_th, d_cnt, d_idx2, d_val2, cap, d_nnz,
                                       d_ws, ws_bytes, nullptr));
    HIP_OK(hipDeviceSynchronize());
    float th2;
    uint64_t cnt2, nnz2[2];
    HIP_OK(hipMemcpy(&th2, d_th, 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(&cnt2, d_cnt, 8, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(nnz2, d_nnz, 16, hipMemcpyDeviceToHost));
    std::vector<uint32_t> idx2(idx.size());
    std::vector<float> val2(idx.size()), res2(n);
    if (std::memcmp(&th2, &th, 4) != 0 || cnt2 != cnt || nnz2[0] != nnz[0] || nnz2[1] != nnz[1]) {
        std::printf("one-call iteration: threshold or counts differ\n");
        return 1;
    }
    HIP_OK(hipMemcpy(idx2.data(), d_idx2, idx2.size() * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(val2.data(), d_val2, val2.size() * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(res2.data(), d_res, n * 4, hipMemcpyDeviceToHost));
    if (idx2 != idx || std::memcmp(val2.data(), val.data(), val.size() * 4) != 0 ||
        std::memcmp(res2.data(), res.data(), n * 4) != 0) {
        std::printf("one-call iteration: selection or residual differs\n");
        return 1;
    }
    std::printf("cabi smoke ok: n=%llu k=%llu selected=%zu region=[%u,%u) reduced=%llu version=%d\n",
                (unsigned long long)n, (unsigned long long)k, idx.size(), lo, hi,
                (unsigned long long)count, okt_version());
    return 0;
}
