// Tile shapes and workspace sizes, shared by the host entry points.
#ifndef OKT_SIZES_H
#define OKT_SIZES_H

#include <stddef.h>
#include <stdint.h>

namespace okt {

// ---- threshold select + compaction ----
// A workgroup of SEL_BLOCK threads owns SEL_WAVES consecutive pieces of the
// vector, one per wave; a wave streams its piece in rounds of 256 elements,
// SEL_U rounds in flight.  The piece length (select_shape below) is never above
// SEL_PIECE_MAX, which keeps the selected entries of a piece inside the wave's
// LDS stash up to a local density of SEL_STASH / SEL_PIECE_MAX = 9.8 %.
constexpr int SEL_BLOCK = 1024;
constexpr int SEL_WAVES = SEL_BLOCK / 64;
constexpr int SEL_U = 4;
// The kernels need more than 64 registers, so a CU holds one workgroup at a time
// anyway: its stash takes nearly the whole LDS (16 waves x 1600 entries x 6 bytes
// = 150 KB of 160).  Gradients select unevenly - whole layers above the
// threshold next to layers with nothing - and a piece that overflows its stash
// is partly walked twice.
constexpr int SEL_STASH = 1600;                // entries per wave
constexpr uint32_t SEL_ROUND = 256u * SEL_U;
constexpr uint32_t SEL_PIECE_MAX = 16384;

struct SelectShape { uint32_t nseg, piece; };
// The select kernels run one 1024-thread workgroup per CU at a time, and a
// workgroup streams for tens of microseconds, so a last round of workgroups that
// fills only part of the chip costs as much as a full one.  The vector is
// therefore cut for whole rounds: `rounds` x `cus` workgroups of equal pieces
// (a multiple of 256 elements, at most SEL_PIECE_MAX), `cus` being the number of
// compute units of the device at hand (device_cus(), never above SEL_CUS_MAX).
constexpr uint32_t SEL_CUS_MAX = 1024;
inline uint64_t select_rounds(uint64_t n, uint32_t cus) {
    const uint64_t per_round = (uint64_t)cus * SEL_WAVES * SEL_PIECE_MAX;
    const uint64_t rounds = (n + per_round - 1) / per_round;
    return rounds ? rounds : 1;
}
inline SelectShape select_shape(uint64_t n, uint32_t cus) {
    const uint64_t waves = (uint64_t)cus * SEL_WAVES * select_rounds(n, cus);
    uint64_t piece = ((n + waves - 1) / waves + 255) / 256 * 256;
    if (piece < SEL_ROUND) piece = SEL_ROUND;
    const uint64_t per_wg = piece * SEL_WAVES;
    return SelectShape{(uint32_t)((n + per_wg - 1) / per_wg), (uint32_t)piece};
}
// Header, segment and group descriptors.  A bound for any device: a launch has at
// most cus x rounds <= n / (SEL_WAVES x SEL_PIECE_MAX) + 1 + cus workgroups.
inline size_t select_ws_bytes(uint64_t n) {
    const uint64_t t = n / ((uint64_t)SEL_WAVES * SEL_PIECE_MAX) + 1 + SEL_CUS_MAX;
    return 64 + 8 * (size_t)(t + (t + 63) / 64);
}

// Vectors longer than the 256 MB last-level cache are read, and where a kernel
// rewrites them densely written, with the non-temporal hint: nothing of them is
// found cached again, and what goes around the cache pushes nothing out.  Shorter
// ones are not: what one kernel writes the next still finds there (the select
// that follows an accumulate, the zeros that follow a refresh iteration's pass).
constexpr uint64_t STREAM_PAST_CACHE_N = 64u << 20;                          // 256 MiB of fp32 and up
inline bool stream_past_cache(uint64_t n) { return n >= STREAM_PAST_CACHE_N; }

// ---- the same through per-tile slots ----
// With a workspace that has room for them, the streaming pass of the selects
// writes what a tile of SLOT_TILE elements (one wave) selects into the tile's own
// slot of SLOT_C entries and counts it; a scan over the counts and a copy out of
// the slots follow as a short second pass, and the tiles that selected more than
// a slot holds (a local density above SLOT_C / SLOT_TILE = 12.5 %) are walked
// again by a third.  Gradients select unevenly - in the layered workloads three
// quarters of the selected entries sit in tiles that select 3 to 12 % - and a
// slot costs address space, not traffic: only the entries written are ever
// touched.  Workspace: a scan state, then per tile a 2-byte count, a 4-byte
// place, 4 bytes of the list of fuller and dense tiles and the slot, as many bytes
// as the vector has elements in all.
constexpr uint32_t SLOT_TILE = 1024;
constexpr uint32_t SLOT_C = 128;
constexpr uint32_t SLOT_GROUP = 4;                   // tiles whose slots are interleaved
constexpr uint32_t SLOT_SCAN_TILES = 1024;           // tiles per workgroup of the second pass and turn
struct SlotPlan {
    uint32_t ntiles;
    uint32_t tpt;                // tiles per thread of the second pass
    uint32_t nseg;               // workgroups of the second pass
    size_t counts_at, place_at, dense_at, slots_at, bytes;   // offsets into the workspace; its size
};
inline size_t round_up_256(size_t v) { return (v + 255) & ~(size_t)255; }
inline SlotPlan slot_plan(uint64_t n, uint32_t cus) {
    SlotPlan p;
    p.ntiles = (uint32_t)((n + SLOT_TILE - 1) / SLOT_TILE);
    // about half as many workgroups as compute units: the pass is short, and every
    // workgroup takes a ticket from one counter
    const uint64_t want = (uint64_t)SLOT_SCAN_TILES * (cus > 1 ? cus / 2 : 1);
    p.tpt = (uint32_t)((p.ntiles + want - 1) / want);
    if (p.tpt == 0) p.tpt = 1;
    if (p.tpt > 63) p.tpt = 63;              // a workgroup's tiles are counted in 16 bits
    const uint64_t per_seg = (uint64_t)SLOT_SCAN_TILES * p.tpt;
    p.nseg = (uint32_t)((p.ntiles + per_seg - 1) / per_seg);
    if (p.nseg == 0) p.nseg = 1;
    // the scan state is sized for the most workgroups any device gives (tpt = 1)
    const uint64_t segs_max = (uint64_t)p.ntiles / SLOT_SCAN_TILES + 1;
    const size_t scan = 64 + 8 * (size_t)(segs_max + (segs_max + 63) / 64);
    p.counts_at = round_up_256(scan);
    p.place_at = p.counts_at + round_up_256(2 * (size_t)p.ntiles);
    p.dense_at = p.place_at + round_up_256(4 * (size_t)p.ntiles);
    p.slots_at = p.dense_at + round_up_256(4 * (size_t)p.ntiles);
    p.bytes = p.slots_at + 8 * (size_t)SLOT_C * ((p.ntiles + SLOT_GROUP - 1) / SLOT_GROUP * SLOT_GROUP);
    return p;
}
inline size_t slot_ws_bytes(uint64_t n) { return slot_plan(n, 256).bytes; }
// Shorter vectors take the one-kernel form: the two extra launches and the scan's
// fixed few microseconds cost more than the leaner streaming pass saves there.
// Measured crossover: the calls that form the accumulator on the way (12 bytes an
// element: the saving is three times the select's) gain from about 40 M elements
// on, the plain selects from about 100 M, where the vector no longer fits the
// last-level cache.
constexpr uint64_t SLOT_MIN_N_SELECT = 96u << 20;
constexpr uint64_t SLOT_MIN_N_ACCUMULATE = 1u << 25;

// ---- index intersection and residual restore ----
constexpr int RST_BLOCK = 256;
constexpr int RST_ROWS = 4;                              // entries per thread
constexpr uint32_t RST_TILE = RST_BLOCK * RST_ROWS;      // local entries per workgroup
constexpr uint32_t RST_WINDOW = 4096;                    // global entries a workgroup stages in LDS
inline uint64_t restore_tiles(uint64_t max_local) {
    return max_local == 0 ? 1 : (max_local + RST_TILE - 1) / RST_TILE;
}
inline size_t restore_ws_bytes(uint64_t max_local) {
    const uint64_t t = restore_tiles(max_local);
    return 64 + 8 * (size_t)(t + (t + 63) / 64);
}

// ---- exact threshold (radix select over the 31-bit magnitude key) ----
constexpr int RS_BITS1 = 11, RS_BITS2 = 11, RS_BITS3 = 9;   // 11 + 11 + 9 = 31
constexpr int RS_MAX_BINS = 1 << 11;
constexpr size_t RS_STATE_BYTES = 256;
constexpr size_t RS_HIST_BYTES = 4 * RS_MAX_BINS * sizeof(uint32_t);   // sample + three digits
constexpr uint64_t RS_SAMPLE_MIN_N = 4u << 20;   // shorter vectors are simply read three times
constexpr uint64_t RS_SAMPLE_BLOCKS = 1024;      // sample: about this many blocks of 1024 elements
inline size_t threshold_ws_min_bytes() { return RS_STATE_BYTES + RS_HIST_BYTES; }
inline size_t threshold_ws_bytes(uint64_t n) {
    // state + histograms + room for the candidate keys (a few percent of the vector)
    return threshold_ws_min_bytes() + 4 * (size_t)(n / 8 + 1024);
}
// A refresh iteration in one pass: the threshold's state and histograms, two scan
// states, candidates with their indices (8 bytes each, a sixteenth of the vector
// and some), and the slots through which a long vector's candidates are
// collected.  A shorter vector takes the three steps one after the other.
inline size_t refresh_scan_bytes(uint64_t n) { return (select_ws_bytes(n) + 255) & ~(size_t)255; }
inline size_t refresh_ws_bytes(uint64_t n) {
    if (n < RS_SAMPLE_MIN_N) return 0;
    return threshold_ws_min_bytes() + 2 * refresh_scan_bytes(n) + 8 * (size_t)(n / 8 + 1024) +
           round_up_256(slot_ws_bytes(n));
}

// ---- sparse reduce ----
// A workgroup of RED_BLOCK threads owns a tile of `slots` consecutive index
// slots of the region and sums into RED_C fp64 accumulators in LDS.  In a region
// that is densely hit a tile is RED_C slots wide and slot = accumulator.  In a
// sparsely hit region a tile is up to RED_S_MAX slots wide: a first sweep marks
// the hit slots in a bitmap, the popcount prefix of the bitmap ranks them, and
// the accumulators are indexed by rank, so the LDS holds hit slots only.
constexpr int RED_BLOCK = 512;
constexpr int RED_UNROLL = 10;                  // blocks of 64 entries a wave keeps in flight (short slices)
constexpr uint32_t RED_C = 4096;                // accumulators per tile and round
constexpr uint32_t RED_S_MAX = 32768;           // widest tile (bits in the bitmap)
constexpr int RED_CHUNKS = 256;                 // contributions handled per sweep

// Two more shapes of the same kernel spend the same LDS differently.  Very
// sparsely hit regions: a wider bitmap paid for with fewer accumulators, so that
// a tile is not cut short by the bitmap with half of its accumulators unused.
// Densely hit regions (accumulator = slot): no rank-to-slot array and a bitmap
// only as wide as the accumulators, which leaves room for more of them.
constexpr uint32_t RED_C_SPARSE = 3840;
constexpr uint32_t RED_S_SPARSE = 49152;
constexpr uint32_t RED_C_DENSE = 6016;                 // a multiple of 32

// Tile shape for a region `width` wide whose union is expected to hold at most
// `expected` entries.  Densely hit (at most RED_C_DENSE / RED_C slots per expected
// entry and accumulator): RED_C_DENSE slots, accumulator = slot, one sweep.  Else
// ranked tiles as wide - any multiple of 32 slots - as keeps the expected number
// of hit slots per tile at RED_FILL of the accumulators: up to RED_S_MAX
// slots with RED_C accumulators, beyond that up to RED_S_SPARSE slots with
// RED_C_SPARSE accumulators.
constexpr double RED_FILL = 0.9;
enum ReduceKind { RED_DENSE = 0, RED_RANKED = 1, RED_SPARSE = 2 };
struct ReduceShape {
    uint32_t slots;
    ReduceKind kind;
};
inline ReduceShape reduce_tile_shape(uint64_t width, uint64_t expected) {
    if (width == 0 || expected == 0)
        return expected == 0 && width > RED_C_DENSE ? ReduceShape{RED_S_SPARSE, RED_SPARSE}
                                                    : ReduceShape{RED_C_DENSE, RED_DENSE};
    const double per_acc = RED_FILL * (double)width / (double)expected;   // slots per accumulator
    const double want = per_acc * RED_C;
    if (want <= RED_C_DENSE) return ReduceShape{RED_C_DENSE, RED_DENSE};
    if (want > RED_S_MAX) {
        const double wide = per_acc * RED_C_SPARSE;
        if (wide >= RED_S_SPARSE) return ReduceShape{RED_S_SPARSE, RED_SPARSE};
        const uint32_t slots = (uint32_t)wide / 32 * 32;
        // narrower than the other shape's widest tile: that one holds more per tile
        return slots > RED_S_MAX ? ReduceShape{slots, RED_SPARSE} : ReduceShape{RED_S_MAX, RED_RANKED};
    }
    return ReduceShape{(uint32_t)want / 32 * 32, RED_RANKED};
}
inline uint64_t reduce_tiles(uint64_t width, uint32_t slots) { return (width + slots - 1) / slots; }
// per region: a 64-byte header, one descriptor per tile and one per 64 tiles,
// then the table of slice starts, (tiles + 1) x P uint32, padded to 64 bytes
inline size_t reduce_ws_bytes_region(uint64_t max_width, uint32_t P, uint32_t slots) {
    uint64_t t = reduce_tiles(max_width, slots);
    if (t == 0) t = 1;
    size_t bytes = 64 + 8 * (size_t)(t + (t + 63) / 64) + 4 * (size_t)(t + 1) * P;
    return (bytes + 63) & ~(size_t)63;
}
inline size_t reduce_ws_bytes(uint64_t B, uint64_t max_width, uint32_t P) {
    return (size_t)B * reduce_ws_bytes_region(max_width, P, RED_C);     // no tile is narrower: largest
}

}  // namespace okt
#endif
