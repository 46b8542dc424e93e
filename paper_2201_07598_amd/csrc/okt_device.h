// Device-side building blocks shared by the okt kernels (gfx950, wave64).
#ifndef OKT_DEVICE_H
#define OKT_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "okt.h"

namespace okt {

constexpr int WAVE = 64;
constexpr uint32_t ABS_MASK = 0x7fffffffu;

// Magnitude key of an fp32: the bit pattern with the sign cleared (Sec. 2:
// top-k is taken by absolute value).
__device__ __forceinline__ uint32_t magnitude_key(float x) {
    return __float_as_uint(x) & ABS_MASK;
}

__device__ __forceinline__ int lane_id() { return (int)__lane_id(); }

// Sum over the 64 lanes of a wave; every lane gets the result.
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
    for (int s = 1; s < WAVE; s <<= 1) v += __shfl_xor(v, s, WAVE);
    return v;
}

// Inclusive prefix sum over the lanes of a wave.
template <typename T>
__device__ __forceinline__ T wave_inclusive_scan(T v) {
    const int lane = lane_id();
#pragma unroll
    for (int s = 1; s < WAVE; s <<= 1) {
        T up = __shfl_up(v, s, WAVE);
        if (lane >= s) v += up;
    }
    return v;
}

// A 16-byte load, optionally with the non-temporal hint.  The hint pays on vectors
// far larger than the last-level cache (nothing of them is found there again:
// 4 to 7 % on the walks below) and costs as much on vectors that fit it, where
// what one iteration writes the next one still finds cached; the host decides by
// the vector's length.
template <bool NT>
__device__ __forceinline__ float4 load_quad(const float4* p) {
    if (NT) {
        typedef float v4f __attribute__((ext_vector_type(4)));
        const v4f v = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
        return make_float4(v.x, v.y, v.z, v.w);
    }
    return *p;
}

// A 16-byte store, optionally with the non-temporal hint: what a streaming kernel
// writes of a vector far larger than the last-level cache is not read again
// before it has been pushed out, and written around the cache it does not push
// out anything else on its way.  Worth 11 to 14 % on the kernels that write the
// residual densely (8 bytes read and 4 written per element) at 110 M elements and
// up, nothing either way at 25 M, where the host does not ask for it.
template <bool NT>
__device__ __forceinline__ void store_quad(float4* p, const float4& v) {
    if (NT) {
        typedef float v4f __attribute__((ext_vector_type(4)));
        const v4f q = {v.x, v.y, v.z, v.w};
        __builtin_nontemporal_store(q, reinterpret_cast<v4f*>(p));
    } else {
        *p = v;
    }
}

// ---------------------------------------------------------------------------
// Chained scan across workgroups (decoupled look-back), two levels deep.
//
// Every tile needs the number of selected entries in all tiles before it.  One
// 64-bit descriptor carries a 2-bit status and a 32-bit count in ONE word, so a
// relaxed device-scope load/store pair is enough: no separate flag, no fence.
// A plain look-back chain advances 64 tiles per round trip through device
// memory (the 8 XCDs do not share an L2), which caps a streaming kernel far
// below HBM speed.  So tiles are grouped by 64: a tile sums the aggregates of
// the earlier tiles of its own group (one round trip) and, at the same time,
// looks back over GROUP descriptors, 64 groups = 4096 tiles per round trip.
// The last tile of a group publishes the group's aggregate and later its
// inclusive prefix.
//
// Tiles are numbered by a ticket taken at workgroup start, so everything a tile
// waits for is published by a workgroup that is already running and that waits
// only for still earlier tickets: every wait ends.  As a backstop each wait is
// bounded; a wait that runs out raises the error word of the workspace header.
// ---------------------------------------------------------------------------
constexpr uint64_t DESC_AGGREGATE = 1ull << 62;   // value = count of this tile / group
constexpr uint64_t DESC_INCLUSIVE = 2ull << 62;   // value = count of groups 0..this
constexpr uint64_t DESC_VALUE = 0xffffffffull;
constexpr int SCAN_GROUP = 64;                    // tiles per group
constexpr uint32_t SPIN_LIMIT = 1u << 24;         // polls before a wait gives up

struct ScanHeader {           // first 64 bytes of the workspace
    uint32_t ticket;
    uint32_t error;           // nonzero: a bounded wait ran out
    uint32_t spin_limit;      // polls a wait may take; 0 = SPIN_LIMIT (set when the state is cleared)
    uint32_t pad[13];
};
constexpr int SCAN_SPIN_WORD = 1;     // the 64-bit word of the header whose low half is spin_limit

__device__ __forceinline__ uint64_t desc_load(const uint64_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void desc_store(uint64_t* p, uint64_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Poll until the descriptor is valid (status != 0).
__device__ __forceinline__ uint64_t desc_wait(const uint64_t* p, ScanHeader* hdr) {
    uint64_t d = desc_load(p);
    uint32_t polls = 0, limit = 0;
    while ((d >> 62) == 0) {
        if (limit == 0) {               // only a wait that has to poll reads the setting
            limit = __hip_atomic_load(&hdr->spin_limit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (limit == 0) limit = SPIN_LIMIT;
        }
        if (++polls > limit) {
            __hip_atomic_store(&hdr->error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return DESC_INCLUSIVE;      // give up: count 0, stops the walk
        }
        __builtin_amdgcn_s_sleep(1);
        d = desc_load(p);
    }
    return d;
}

// Called by ONE full wave.  Publishes the aggregate of `tile` and returns the sum
// of the aggregates of the earlier tiles of its group (to every lane).  If the
// tile closes its group, also publishes the group's aggregate.
__device__ __forceinline__ uint32_t scan_within_group(ScanHeader* hdr, uint64_t* tile_desc,
                                                      uint64_t* group_desc, uint32_t tile,
                                                      uint32_t aggregate) {
    const int lane = lane_id();
    const uint32_t g = tile / SCAN_GROUP, j = tile % SCAN_GROUP;
    // storing the same word twice is harmless: a caller may have published early
    if (lane == 0) desc_store(tile_desc + tile, DESC_AGGREGATE | aggregate);
    uint32_t v = 0;
    if ((uint32_t)lane < j) v = (uint32_t)(desc_wait(tile_desc + g * SCAN_GROUP + lane, hdr) & DESC_VALUE);
    const uint32_t before = wave_sum(v);
    if (j == SCAN_GROUP - 1 && lane == 0)
        desc_store(group_desc + g, (g == 0 ? DESC_INCLUSIVE : DESC_AGGREGATE) | (uint64_t)(before + aggregate));
    return before;
}

// A tile may publish its aggregate as soon as it knows it, ahead of the scan.
__device__ __forceinline__ void scan_publish_early(uint64_t* tile_desc, uint32_t tile,
                                                   uint32_t aggregate) {
    desc_store(tile_desc + tile, DESC_AGGREGATE | aggregate);
}

// Called by ONE full wave.  Returns the count of all groups before group g.
__device__ __forceinline__ uint32_t scan_across_groups(ScanHeader* hdr, const uint64_t* group_desc,
                                                       uint32_t g) {
    const int lane = lane_id();
    uint32_t exclusive = 0;
    int64_t base = (int64_t)g - 1;
    while (base >= 0) {
        const int64_t t = base - lane;
        uint64_t d = DESC_INCLUSIVE;              // before group 0: nothing
        if (t >= 0) d = desc_wait(group_desc + t, hdr);
        const uint64_t inclusive_lanes = __ballot((d >> 62) == 2);
        const uint32_t v = (uint32_t)(d & DESC_VALUE);
        if (inclusive_lanes != 0) {
            const int first = __ffsll((unsigned long long)inclusive_lanes) - 1;
            exclusive += wave_sum(lane <= first ? v : 0u);
            break;
        }
        exclusive += wave_sum(v);
        base -= WAVE;
    }
    return exclusive;
}

// Thread 0 of the tile that closes group g (g > 0) calls this once the group's
// exclusive prefix is known.
__device__ __forceinline__ void scan_close_group(uint64_t* group_desc, uint32_t g,
                                                 uint32_t inclusive) {
    desc_store(group_desc + g, DESC_INCLUSIVE | (uint64_t)inclusive);
}

// Workspace of a chained scan: the header, one descriptor per tile, then one per
// group.
constexpr size_t SCAN_HEADER_BYTES = sizeof(ScanHeader);
static_assert(SCAN_HEADER_BYTES == 64, "header is one 64-byte line");
inline uint64_t scan_groups(uint64_t tiles) { return (tiles + SCAN_GROUP - 1) / SCAN_GROUP; }
inline size_t scan_ws_bytes(uint64_t tiles) {
    return SCAN_HEADER_BYTES + 8 * (size_t)(tiles + scan_groups(tiles));
}

// Clear the `words` 64-bit words of a scan state (header and descriptors) and set
// the header's spin limit (a fill kernel rather than a memset node, so that a
// caller may capture the calls into a HIP graph).
__global__ void clear_scan_state_kernel(uint64_t* p, uint64_t words, uint32_t spin_limit);

hipError_t launch_clear_scan_state(void* p, uint64_t words, hipStream_t stream);

// Polls a bounded wait may take before it gives up, as set by
// okt_debug_spin_limit (0 = SPIN_LIMIT).
uint32_t spin_limit_setting();

// Compute units of the calling thread's current device, asked of the runtime once
// per device and kept (host side, no allocation); 256 where there is no device
// to ask, never above 1024.  Sizes the launches that want one workgroup per CU.
uint32_t device_cus();

// Status of the launches an entry point has just made: OKT_OK, or OKT_ERR_HIP
// with the runtime's error kept for okt_last_hip_error.
int launch_status();
int launch_failed(hipError_t e);

// Measurement hook (okt_time_next_kernel): record the pending pair of events, if
// any, right before and right after the launch of a call's main kernel.
void timing_before(hipStream_t stream);
void timing_after(hipStream_t stream);

// Measurement only (okt_ceiling.hip): one workgroup per tile of the sparse
// reduce, reading the tile's slices through the reduce's own slice table and
// writing every entry once; no sums, no ranks, no scan.
__global__ void gather_ceiling_kernel(const uint32_t* idx_cat, const float* val_cat,
                                      const uint64_t* seg_begin, uint32_t seg_stride,
                                      const uint32_t* lo_hi, uint32_t P, uint32_t max_width,
                                      uint32_t slots, uint32_t* idx_out, float* val_out,
                                      uint64_t capacity, const char* ws, uint32_t ws_region_bytes,
                                      uint32_t table_offset);

inline bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

}  // namespace okt
#endif
