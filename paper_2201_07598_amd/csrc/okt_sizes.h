// Tile shapes and workspace sizes, shared by the host entry points.
#ifndef OKT_SIZES_H
#define OKT_SIZES_H

#include <stddef.h>
#include <stdint.h>

namespace okt {

// ---- threshold select + compaction ----
constexpr int SEL_BLOCK = 256;                 // threads per workgroup
constexpr int SEL_ITERS = 4;                   // float4 loads per thread
constexpr int SEL_TILE = SEL_BLOCK * SEL_ITERS * 4;

inline uint64_t select_tiles(uint64_t n) { return (n + SEL_TILE - 1) / SEL_TILE; }
inline size_t select_ws_bytes(uint64_t n) { return 64 + 8 * (size_t)select_tiles(n); }

// ---- exact threshold (radix select over the 31-bit magnitude key) ----
constexpr int RS_BITS1 = 11, RS_BITS2 = 11, RS_BITS3 = 9;   // 11 + 11 + 9 = 31
constexpr int RS_MAX_BINS = 1 << 11;
constexpr size_t RS_STATE_BYTES = 256;
constexpr size_t RS_HIST_BYTES = 3 * RS_MAX_BINS * sizeof(uint32_t);
inline size_t threshold_ws_min_bytes() { return RS_STATE_BYTES + RS_HIST_BYTES; }
inline size_t threshold_ws_bytes(uint64_t n) {
    // state + three histograms + room for the keys that survive the first digit
    return threshold_ws_min_bytes() + 4 * (size_t)(n / 8 + 1024);
}

// ---- sparse reduce ----
constexpr int RED_BLOCK = 256;
constexpr int RED_TILE = 4096;                 // index slots per workgroup
constexpr int RED_CHUNKS = 1024;               // contributions handled per sweep
inline uint64_t reduce_tiles(uint64_t width) { return (width + RED_TILE - 1) / RED_TILE; }
// per region: a 64-byte header (ticket) and one descriptor per tile
inline size_t reduce_ws_bytes_region(uint64_t max_width) {
    uint64_t t = reduce_tiles(max_width);
    if (t == 0) t = 1;
    return 64 + 8 * (size_t)t;
}
inline size_t reduce_ws_bytes(uint64_t B, uint64_t max_width) {
    return (size_t)B * reduce_ws_bytes_region(max_width);
}

}  // namespace okt
#endif
