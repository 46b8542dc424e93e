// Host-side pieces of the C ABI that belong to no single kernel.
#include "okt_device.h"
#include "okt_sizes.h"

#include <atomic>

namespace okt {

static thread_local hipError_t g_last_hip_error = hipSuccess;

int launch_failed(hipError_t e) {
    g_last_hip_error = e;
    return OKT_ERR_HIP;
}

int launch_status() {
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? OKT_OK : launch_failed(e);
}

static thread_local hipEvent_t g_time_start = nullptr, g_time_stop = nullptr;

void timing_before(hipStream_t stream) {
    if (g_time_start) (void)hipEventRecord(g_time_start, stream);
    g_time_start = nullptr;
}
void timing_after(hipStream_t stream) {
    if (g_time_stop) (void)hipEventRecord(g_time_stop, stream);
    g_time_stop = nullptr;
}

uint32_t device_cus() {
    constexpr int MAX_DEVICES = 64;
    constexpr uint32_t FALLBACK = 256;
    static std::atomic<uint32_t> known[MAX_DEVICES];     // zero-initialised: not asked yet
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        (void)hipGetLastError();                         // no device is not a launch error
        return FALLBACK;
    }
    uint32_t cus = known[dev].load(std::memory_order_relaxed);
    if (cus == 0) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) {
            (void)hipGetLastError();
            v = (int)FALLBACK;
        }
        cus = (uint32_t)v > SEL_CUS_MAX ? SEL_CUS_MAX : (uint32_t)v;
        known[dev].store(cus, std::memory_order_relaxed);
    }
    return cus;
}

static std::atomic<uint32_t> g_spin_limit{0};
uint32_t spin_limit_setting() { return g_spin_limit.load(std::memory_order_relaxed); }

__global__ void clear_scan_state_kernel(uint64_t* p, uint64_t words, uint32_t spin_limit) {
    uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (; i < words; i += stride) p[i] = i == SCAN_SPIN_WORD ? (uint64_t)spin_limit : 0ull;
}

hipError_t launch_clear_scan_state(void* p, uint64_t words, hipStream_t stream) {
    if (words == 0) return hipSuccess;
    uint64_t blocks = (words + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(clear_scan_state_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                       (uint64_t*)p, words, spin_limit_setting());
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) launch_failed(e);
    return e;
}

}  // namespace okt

extern "C" {

const char* okt_last_hip_error(void) { return hipGetErrorString(okt::g_last_hip_error); }

void okt_debug_spin_limit(uint32_t polls) {
    okt::g_spin_limit.store(polls, std::memory_order_relaxed);
}

void okt_time_next_kernel(void* start_event, void* stop_event) {
    okt::g_time_start = (hipEvent_t)start_event;
    okt::g_time_stop = (hipEvent_t)stop_event;
}

const char* okt_status_string(int status) {
    switch (status) {
        case OKT_OK: return "ok";
        case OKT_ERR_INVALID_ARG: return "invalid argument";
        case OKT_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case OKT_ERR_HIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

int okt_version(void) { return 100; }

size_t okt_workspace_bytes(uint64_t n_max, uint32_t P_max) {
    if (P_max == 0) P_max = 1;
    size_t need = okt::threshold_ws_bytes(n_max);
    size_t s = okt::select_ws_bytes(n_max);
    if (s > need) need = s;
    s = okt::refresh_ws_bytes(n_max);
    if (s > need) need = s;
    s = okt::restore_ws_bytes(n_max);
    if (s > need) need = s;
    s = okt::reduce_ws_bytes(1, n_max, P_max);
    if (s > need) need = s;
    return (need + 255) & ~(size_t)255;
}

size_t okt_sparse_reduce_batch_workspace_bytes(uint32_t B, uint32_t P, uint32_t max_width) {
    return (okt::reduce_ws_bytes(B, max_width, P ? P : 1) + 255) & ~(size_t)255;
}

}  // extern "C"
