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

// ---------------------------------------------------------------------------
// Chained scan across workgroups (decoupled look-back).  One 64-bit descriptor
// per tile carries a 2-bit status and a 32-bit count in ONE word, so a relaxed
// device-scope load/store pair is enough: no separate flag, no fence.  Tiles
// are numbered by a ticket taken at workgroup start, so every predecessor of a
// tile belongs to a workgroup that is already running; the spin below therefore
// always ends.
// ---------------------------------------------------------------------------
constexpr uint64_t DESC_AGGREGATE = 1ull << 62;   // value = count of this tile
constexpr uint64_t DESC_INCLUSIVE = 2ull << 62;   // value = count of tiles 0..this
constexpr uint64_t DESC_VALUE = 0xffffffffull;

__device__ __forceinline__ uint64_t desc_load(const uint64_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void desc_store(uint64_t* p, uint64_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Called by ONE full wave of the workgroup that owns `tile`.  Publishes the
// tile's count and returns the sum of the counts of tiles 0..tile-1 (to every
// lane).  desc[] must be zero before the first tile starts.
__device__ __forceinline__ uint32_t lookback_exclusive(uint64_t* desc, uint32_t tile,
                                                       uint32_t aggregate) {
    const int lane = lane_id();
    if (tile == 0) {
        if (lane == 0) desc_store(desc, DESC_INCLUSIVE | aggregate);
        return 0;
    }
    if (lane == 0) desc_store(desc + tile, DESC_AGGREGATE | aggregate);
    uint32_t exclusive = 0;
    int64_t base = (int64_t)tile - 1;
    for (;;) {
        const int64_t t = base - lane;
        uint64_t d = DESC_INCLUSIVE;             // tiles before 0: nothing
        if (t >= 0) {
            d = desc_load(desc + t);
            while ((d >> 62) == 0) {
                __builtin_amdgcn_s_sleep(1);
                d = desc_load(desc + t);
            }
        }
        const uint64_t inclusive_lanes = __ballot((d >> 62) == 2);
        uint32_t v = (uint32_t)(d & DESC_VALUE);
        if (inclusive_lanes != 0) {
            const int first = __ffsll((unsigned long long)inclusive_lanes) - 1;
            exclusive += wave_sum(lane <= first ? v : 0u);
            break;
        }
        exclusive += wave_sum(v);
        base -= WAVE;
    }
    if (lane == 0) desc_store(desc + tile, DESC_INCLUSIVE | (uint64_t)(exclusive + aggregate));
    return exclusive;
}

// Workspace header used by the chained scans: a ticket counter, then the
// descriptors.  Kept on its own 64 bytes.
constexpr size_t SCAN_HEADER_BYTES = 64;

// Zero `words` 64-bit words (a fill kernel rather than a memset node, so that a
// caller may capture the calls into a HIP graph).
__global__ void zero_words_kernel(uint64_t* p, uint64_t words);

hipError_t launch_zero_words(void* p, uint64_t words, hipStream_t stream);

inline bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

}  // namespace okt
#endif
