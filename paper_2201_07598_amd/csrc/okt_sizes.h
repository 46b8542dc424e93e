// Tile shapes and workspace sizes, shared by the host entry points.
#ifndef OKT_SIZES_H
#define OKT_SIZES_H

#include <stddef.h>
#include <stdint.h>

namespace okt {

// ---- threshold select + compaction ----
// A workgroup of SEL_BLOCK threads owns SEL_WAVES consecutive pieces of the
// vector, one per wave; a wave streams its piece in rounds of 256 elements,
// SEL_U rounds in flight.  The piece length is chosen so that about
// SEL_TARGET_WGS workgroups (32 waves per CU on 256 CUs) cover the vector, but never
// above SEL_PIECE_MAX, which keeps the selected entries of a piece inside the
// wave's LDS stash up to a density of SEL_STASH / SEL_PIECE_MAX = 3.7 %.
#ifndef OKT_SEL_U
#define OKT_SEL_U 4
#endif
#ifndef OKT_SEL_TICKET
#define OKT_SEL_TICKET true
#endif
#ifndef OKT_SEL_TARGET_WGS
#define OKT_SEL_TARGET_WGS 512
#endif
#ifndef OKT_SEL_BLOCK
#define OKT_SEL_BLOCK 1024
#endif
constexpr int SEL_BLOCK = OKT_SEL_BLOCK;
constexpr int SEL_WAVES = SEL_BLOCK / 64;
constexpr int SEL_U = OKT_SEL_U;
constexpr int SEL_STASH = 608;                 // entries per wave: 32 waves fit one CU's LDS
constexpr bool SEL_TICKET = OKT_SEL_TICKET;    // false: measurement builds only
constexpr uint32_t SEL_ROUND = 256u * SEL_U;
constexpr uint32_t SEL_PIECE_MAX = 16384;
constexpr uint32_t SEL_TARGET_WGS = OKT_SEL_TARGET_WGS;

struct SelectShape { uint32_t nseg, piece; };
inline SelectShape select_shape(uint64_t n) {
    uint64_t per_wave = (n + (uint64_t)SEL_TARGET_WGS * SEL_WAVES - 1) / ((uint64_t)SEL_TARGET_WGS * SEL_WAVES);
    uint64_t piece = (per_wave + SEL_ROUND - 1) / SEL_ROUND * SEL_ROUND;
    if (piece < SEL_ROUND) piece = SEL_ROUND;
    if (piece > SEL_PIECE_MAX) piece = SEL_PIECE_MAX;
    const uint64_t per_wg = piece * SEL_WAVES;
    return SelectShape{(uint32_t)((n + per_wg - 1) / per_wg), (uint32_t)piece};
}
inline size_t select_ws_bytes(uint64_t n) {       // header, segment and group descriptors
    const uint64_t t = select_shape(n).nseg;
    return 64 + 8 * (size_t)(t + (t + 63) / 64);
}

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
// per region: a 64-byte header, one descriptor per tile and one per 64 tiles
inline size_t reduce_ws_bytes_region(uint64_t max_width) {
    uint64_t t = reduce_tiles(max_width);
    if (t == 0) t = 1;
    return 64 + 8 * (size_t)(t + (t + 63) / 64);
}
inline size_t reduce_ws_bytes(uint64_t B, uint64_t max_width) {
    return (size_t)B * reduce_ws_bytes_region(max_width);
}

}  // namespace okt
#endif
