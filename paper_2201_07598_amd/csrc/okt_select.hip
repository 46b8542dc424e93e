// okt_threshold_select: threshold top-k selection, packaging into a consecutive
// sorted COO buffer, and zeroing of the selected residual entries, in ONE pass
// over acc (Sec. 3.1.3 threshold selection; Sec. 3.1.2 packaging; Algorithm 2,
// line 6 residual update).
//
// HBM-bound: 4 B read per element plus 12 B per selected entry (index, value,
// zero).  The vector is cut into contiguous pieces, one per wave; a wave streams
// its piece with 16-byte loads (1 KiB contiguous per load instruction, several
// in flight) and ranks the selected elements with wave ballots, so the hot loop
// has no barrier and no wait.  The place of a workgroup's entries in the output
// comes from a two-level chained scan over workgroup counts (decoupled
// look-back), so acc is read exactly once.
#include "okt_select_kernel.h"
#include "okt_sizes.h"
#include "okt_slots.h"

#include <atomic>
#include <mutex>

// Scan state of okt_threshold_select_noalloc: device memory that belongs to the
// library, one copy per GPU, held until the process ends.  Host code never uses
// this name as an address; it asks the runtime where the array lives on the
// current device (static_scratch below) and passes that pointer on.
static __device__ __align__(256) unsigned char scratch[OKT_SELECT_NOALLOC_SCRATCH_BYTES];

namespace okt {

__global__ void select_empty_kernel(uint64_t* nnz_out) {
    nnz_out[0] = 0;
    nnz_out[1] = 0;
}

}  // namespace okt

namespace okt {

// Argument errors of the dense select, found before anything is launched.
static int dense_select_args(const float* d_acc, uint64_t n, const float* d_threshold,
                             const uint32_t* d_idx_out, const float* d_val_out, uint64_t capacity,
                             const uint64_t* d_nnz_out) {
    if (!d_nnz_out || !aligned(d_nnz_out, 8)) return OKT_ERR_INVALID_ARG;
    if (n > 0xffffffffull) return OKT_ERR_INVALID_ARG;
    if (n == 0) return OKT_OK;
    if (!d_acc || !d_threshold || !aligned(d_acc, 16) || !aligned(d_threshold, 4))
        return OKT_ERR_INVALID_ARG;
    if (capacity > 0 && (!d_idx_out || !d_val_out || !aligned(d_idx_out, 4) ||
                         !aligned(d_val_out, 4)))
        return OKT_ERR_INVALID_ARG;
    return OKT_OK;
}

// Shortest vector that takes the slot path (okt_debug_slot_min_n; 0 = built in).
static std::atomic<uint64_t> g_slot_min_n{0};
uint64_t slot_min_n(bool accumulating) {
    const uint64_t set = g_slot_min_n.load(std::memory_order_relaxed);
    return set ? set : accumulating ? SLOT_MIN_N_ACCUMULATE : SLOT_MIN_N_SELECT;
}
static bool slots_apply(uint64_t n, size_t ws_bytes, bool accumulating) {
    return n >= slot_min_n(accumulating) && ws_bytes >= slot_ws_bytes(n);
}

int launch_slot_finish(float* d_acc, uint64_t n, const float* d_threshold, const SlotPlan& plan,
                       char* ws, int after, bool dense_zero, uint32_t* d_idx_out, float* d_val_out,
                       uint64_t capacity, uint64_t* d_nnz_out, hipStream_t s) {
    ScanHeader* hdr = (ScanHeader*)ws;
    uint64_t* seg_desc = (uint64_t*)(ws + SCAN_HEADER_BYTES);
    uint64_t* group_desc = seg_desc + plan.nseg;
    const uint16_t* counts = (const uint16_t*)(ws + plan.counts_at);
    uint32_t* place = (uint32_t*)(ws + plan.place_at);
    const SlotEntry* slots = (const SlotEntry*)(ws + plan.slots_at);
    uint32_t* dense_list = (uint32_t*)(ws + plan.dense_at);
    hipLaunchKernelGGL(slot_scan_kernel<SLOT_SCAN_BLOCK>, dim3(plan.nseg), dim3(SLOT_SCAN_BLOCK), 0, s, counts, place,
                       dense_list, plan.ntiles, plan.tpt, capacity, d_nnz_out, hdr, seg_desc,
                       group_desc, plan.nseg);
    // a lane per tile, and at least a full load of waves on every compute unit for the
    // dense tiles, which are shared out over all the waves of the launch
    constexpr uint32_t per_wg = (SLOT_EMIT_BLOCK / WAVE) * SLOT_EMIT_TILES;
    uint32_t grid = (plan.ntiles + per_wg - 1) / per_wg;
    if (grid < 8 * device_cus()) grid = 8 * device_cus();
    auto* emit = after == SLOT_ZERO      ? slot_emit_kernel<SLOT_ZERO, true>
                 : after == SLOT_RESTORE ? slot_emit_kernel<SLOT_RESTORE, true>
                 : dense_zero            ? slot_emit_kernel<SLOT_KEEP, true>
                                         : slot_emit_kernel<SLOT_KEEP, false>;
    hipLaunchKernelGGL(emit, dim3(grid), dim3(SLOT_EMIT_BLOCK), 0, s, d_acc, (uint32_t)n, d_threshold,
                       counts, place, slots, dense_list, hdr, plan.ntiles, d_idx_out, d_val_out,
                       capacity);
    return launch_status();
}

// The dense select, with (Source = DenseSource) or without (DenseCopySource) the
// zeroing of the emitted entries.
template <typename Source>
static int launch_dense_select(float* d_acc, uint64_t n, const float* d_threshold,
                               uint32_t* d_idx_out, float* d_val_out, uint64_t capacity,
                               uint64_t* d_nnz_out, void* d_ws, size_t ws_bytes, hipStream_t s) {
    const int args = dense_select_args(d_acc, n, d_threshold, d_idx_out, d_val_out, capacity,
                                       d_nnz_out);
    if (args != OKT_OK) return args;
    if (n == 0) {
        hipLaunchKernelGGL(select_empty_kernel, dim3(1), dim3(1), 0, s, d_nnz_out);
        return launch_status();
    }
    const SelectShape shape = select_shape(n, device_cus());
    if (!d_ws || !aligned(d_ws, 256) || ws_bytes < select_ws_bytes(n)) return OKT_ERR_WORKSPACE;
    if (slots_apply(n, ws_bytes, false)) {
        const SlotPlan plan = slot_plan(n, device_cus());
        char* ws = (char*)d_ws;
        timing_before(s);
        constexpr bool zero = std::is_same<Source, DenseSource>::value;
        auto* fill = stream_past_cache(n) ? slot_fill_kernel<true> : slot_fill_kernel<false>;
        constexpr uint32_t per_wg = SLOT_FILL_BLOCK / WAVE;
        hipLaunchKernelGGL(fill, dim3((plan.ntiles + per_wg - 1) / per_wg), dim3(SLOT_FILL_BLOCK), 0,
                           s, d_acc, (uint32_t)n, d_threshold, (uint16_t*)(ws + plan.counts_at),
                           (SlotEntry*)(ws + plan.slots_at), plan.ntiles, (uint64_t*)ws,
                           (uint32_t)(scan_ws_bytes(plan.nseg) / 8), spin_limit_setting());
        timing_after(s);
        return launch_slot_finish(d_acc, n, d_threshold, plan, ws, zero ? SLOT_ZERO : SLOT_KEEP,
                                  zero, d_idx_out, d_val_out, capacity, d_nnz_out, s);
    }
    ScanHeader* hdr = (ScanHeader*)d_ws;
    uint64_t* seg_desc = (uint64_t*)((char*)d_ws + SCAN_HEADER_BYTES);
    uint64_t* group_desc = seg_desc + shape.nseg;
    if (launch_clear_scan_state(d_ws, scan_ws_bytes(shape.nseg) / 8, s) != hipSuccess)
        return OKT_ERR_HIP;
    timing_before(s);
    auto* kernel = stream_past_cache(n) ? select_kernel<SEL_BLOCK, SEL_U, SEL_STASH, Source, true>
                                        : select_kernel<SEL_BLOCK, SEL_U, SEL_STASH, Source, false>;
    hipLaunchKernelGGL(kernel, dim3(shape.nseg), dim3(SEL_BLOCK), 0, s, d_acc, (uint32_t)n, d_threshold,
                       d_idx_out, d_val_out, capacity, d_nnz_out, hdr, seg_desc, group_desc,
                       shape.nseg, shape.piece);
    timing_after(s);
    return launch_status();
}

}  // namespace okt

extern "C" void okt_debug_slot_min_n(uint64_t n) {
    okt::g_slot_min_n.store(n, std::memory_order_relaxed);
}

extern "C" uint64_t okt_slot_min_n(int accumulating) { return okt::slot_min_n(accumulating != 0); }

extern "C" int okt_threshold_select(float* d_acc_inout, uint64_t n, const float* d_threshold,
                                    uint32_t* d_idx_out, float* d_val_out, uint64_t capacity,
                                    uint64_t* d_nnz_out, void* d_ws, size_t ws_bytes,
                                    void* stream) {
    return okt::launch_dense_select<okt::DenseSource>(d_acc_inout, n, d_threshold, d_idx_out,
                                                      d_val_out, capacity, d_nnz_out, d_ws,
                                                      ws_bytes, (hipStream_t)stream);
}

namespace okt {

// Address of `scratch` on the calling thread's current device, looked up once per
// device and kept.
static int static_scratch(void** out) {
    constexpr int MAX_DEVICES = 64;
    static std::mutex guard;
    static void* where[MAX_DEVICES] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return launch_failed(e);
    if (dev < 0 || dev >= MAX_DEVICES) return OKT_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(guard);
    if (!where[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return launch_failed(e);
        if (!p) return launch_failed(hipErrorInvalidSymbol);
        where[dev] = p;
    }
    *out = where[dev];
    return OKT_OK;
}

}  // namespace okt

extern "C" int okt_threshold_select_noalloc(float* d_acc_inout, uint64_t n,
                                            const float* d_threshold, uint32_t* d_idx_out,
                                            float* d_val_out, uint64_t capacity,
                                            uint64_t* d_nnz_out, void* stream) {
    const int args = okt::dense_select_args(d_acc_inout, n, d_threshold, d_idx_out, d_val_out,
                                            capacity, d_nnz_out);
    if (args != OKT_OK) return args;
    // more workgroups than the array has descriptors for: refuse before anything runs
    if (okt::select_ws_bytes(n) > sizeof(scratch)) return OKT_ERR_WORKSPACE;
    void* ws = nullptr;
    if (n != 0) {                      // an empty vector needs no scan state
        const int rc = okt::static_scratch(&ws);
        if (rc != OKT_OK) return rc;
    }
    // the launches of okt_threshold_select's one-kernel form (the array is too small
    // for slots at any length that would take the other): a fill kernel that clears
    // the scan state (the array keeps what the last call left), then the select kernel
    return okt::launch_dense_select<okt::DenseSource>(d_acc_inout, n, d_threshold, d_idx_out,
                                                      d_val_out, capacity, d_nnz_out, ws,
                                                      sizeof(scratch), (hipStream_t)stream);
}

extern "C" int okt_threshold_select_copy(const float* d_acc, uint64_t n, const float* d_threshold,
                                         uint32_t* d_idx_out, float* d_val_out,
                                         uint64_t capacity, uint64_t* d_nnz_out, void* d_ws,
                                         size_t ws_bytes, void* stream) {
    // DenseCopySource never writes through the pointer
    return okt::launch_dense_select<okt::DenseCopySource>(
        const_cast<float*>(d_acc), n, d_threshold, d_idx_out, d_val_out, capacity, d_nnz_out, d_ws,
        ws_bytes, (hipStream_t)stream);
}

extern "C" int okt_accumulate_select(const float* d_grad, float* d_residual_inout, float lr,
                                     uint64_t n, const float* d_threshold, uint32_t* d_idx_out,
                                     float* d_val_out, uint64_t capacity, uint64_t* d_nnz_out,
                                     void* d_ws, size_t ws_bytes, void* stream) {
    using namespace okt;
    hipStream_t s = (hipStream_t)stream;
    if (!d_nnz_out || !aligned(d_nnz_out, 8)) return OKT_ERR_INVALID_ARG;
    if (n > 0xffffffffull) return OKT_ERR_INVALID_ARG;
    if (n == 0) {
        hipLaunchKernelGGL(select_empty_kernel, dim3(1), dim3(1), 0, s, d_nnz_out);
        return launch_status();
    }
    if (!d_grad || !d_residual_inout || !d_threshold || d_grad == d_residual_inout ||
        !aligned(d_grad, 16) || !aligned(d_residual_inout, 16) || !aligned(d_threshold, 4))
        return OKT_ERR_INVALID_ARG;
    if (capacity > 0 && (!d_idx_out || !d_val_out || !aligned(d_idx_out, 4) ||
                         !aligned(d_val_out, 4)))
        return OKT_ERR_INVALID_ARG;
    const SelectShape shape = select_shape(n, device_cus());
    if (!d_ws || !aligned(d_ws, 256) || ws_bytes < select_ws_bytes(n)) return OKT_ERR_WORKSPACE;
    if (slots_apply(n, ws_bytes, true)) {
        const SlotPlan plan = slot_plan(n, device_cus());
        char* ws = (char*)d_ws;
        timing_before(s);
        auto* fill = stream_past_cache(n) ? slot_fill_accumulate_kernel<true, true>
                                          : slot_fill_accumulate_kernel<true, false>;
        constexpr uint32_t per_wg = SLOT_FILL_BLOCK / WAVE;
        hipLaunchKernelGGL(fill, dim3((plan.ntiles + per_wg - 1) / per_wg), dim3(SLOT_FILL_BLOCK), 0,
                           s, d_grad, d_residual_inout, lr, (uint32_t)n, d_threshold,
                           (uint16_t*)(ws + plan.counts_at), (SlotEntry*)(ws + plan.slots_at),
                           plan.ntiles, (uint64_t*)ws, (uint32_t)(scan_ws_bytes(plan.nseg) / 8),
                           spin_limit_setting());
        timing_after(s);
        return launch_slot_finish(d_residual_inout, n, d_threshold, plan, ws, SLOT_RESTORE, true,
                                  d_idx_out, d_val_out, capacity, d_nnz_out, s);
    }
    ScanHeader* hdr = (ScanHeader*)d_ws;
    uint64_t* seg_desc = (uint64_t*)((char*)d_ws + SCAN_HEADER_BYTES);
    uint64_t* group_desc = seg_desc + shape.nseg;
    if (launch_clear_scan_state(d_ws, scan_ws_bytes(shape.nseg) / 8, s) != hipSuccess)
        return OKT_ERR_HIP;
    timing_before(s);
    auto* kernel = stream_past_cache(n) ? accumulate_select_kernel<SEL_BLOCK, SEL_U, SEL_STASH, true>
                                        : accumulate_select_kernel<SEL_BLOCK, SEL_U, SEL_STASH, false>;
    hipLaunchKernelGGL(kernel, dim3(shape.nseg), dim3(SEL_BLOCK), 0, s, d_grad, d_residual_inout, lr,
                       (uint32_t)n, d_threshold, d_idx_out, d_val_out, capacity, d_nnz_out, hdr,
                       seg_desc, group_desc, shape.nseg, shape.piece);
    timing_after(s);
    return launch_status();
}

extern "C" int okt_coo_threshold_select(const uint32_t* d_idx_in, const float* d_val_in,
                                        const uint64_t* d_nnz_in, uint64_t max_nnz,
                                        const float* d_threshold, uint32_t* d_idx_out,
                                        float* d_val_out, uint64_t capacity, uint64_t* d_nnz_out,
                                        void* d_ws, size_t ws_bytes, void* stream) {
    using namespace okt;
    hipStream_t s = (hipStream_t)stream;
    if (!d_nnz_out || !aligned(d_nnz_out, 8)) return OKT_ERR_INVALID_ARG;
    if (max_nnz > 0xffffffffull) return OKT_ERR_INVALID_ARG;
    if (max_nnz == 0) {
        hipLaunchKernelGGL(select_empty_kernel, dim3(1), dim3(1), 0, s, d_nnz_out);
        return launch_status();
    }
    if (!d_idx_in || !d_val_in || !d_nnz_in || !d_threshold || !aligned(d_idx_in, 4) ||
        !aligned(d_val_in, 16) || !aligned(d_nnz_in, 8) || !aligned(d_threshold, 4))
        return OKT_ERR_INVALID_ARG;
    if (capacity > 0 && (!d_idx_out || !d_val_out || !aligned(d_idx_out, 4) ||
                         !aligned(d_val_out, 4)))
        return OKT_ERR_INVALID_ARG;
    const SelectShape shape = select_shape(max_nnz, device_cus());
    if (!d_ws || !aligned(d_ws, 256) || ws_bytes < select_ws_bytes(max_nnz))
        return OKT_ERR_WORKSPACE;
    ScanHeader* hdr = (ScanHeader*)d_ws;
    uint64_t* seg_desc = (uint64_t*)((char*)d_ws + SCAN_HEADER_BYTES);
    uint64_t* group_desc = seg_desc + shape.nseg;
    if (launch_clear_scan_state(d_ws, scan_ws_bytes(shape.nseg) / 8, s) != hipSuccess)
        return OKT_ERR_HIP;
    timing_before(s);
    hipLaunchKernelGGL((coo_select_kernel<SEL_BLOCK, SEL_U, SEL_STASH>),
                       dim3(shape.nseg), dim3(SEL_BLOCK), 0, s, d_idx_in, d_val_in, d_nnz_in,
                       (uint32_t)max_nnz, d_threshold, d_idx_out, d_val_out, capacity, d_nnz_out,
                       hdr, seg_desc, group_desc, shape.nseg, shape.piece);
    timing_after(s);
    return launch_status();
}
