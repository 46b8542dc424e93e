// Host check of the workspace arithmetic in okt_sizes.h: for vector lengths from 1
// to 2^32 - 1 and devices of 1 to 1024 compute units, the layout of the
// three-pass select (scan state, counts, places, list, slots) is in order, does
// not overlap, covers every tile, stays inside what okt_workspace_bytes-style
// bounds promise for any device, and the second pass's shape (tiles per thread,
// workgroups) covers all tiles within the limits its kernel assumes.  Prints the
// number of cases and exits 0, or the first violations and exits 1.
#include <cstdint>
#include <cstdio>
#include <random>

#include "okt_sizes.h"

int main() {
    using namespace okt;
    std::mt19937_64 rng(2201);
    long bad = 0, cases = 0;
    auto fail = [&](const char* what, uint64_t n, uint32_t cus) {
        if (bad < 8) std::printf("n=%llu cus=%u: %s\n", (unsigned long long)n, cus, what);
        ++bad;
    };
    const uint32_t cu_counts[] = {1, 2, 3, 7, 64, 104, 128, 228, 256, 304, 1000, 1024};
    for (int rep = 0; rep < 200000; ++rep) {
        uint64_t n;
        switch (rng() % 5) {
            case 0: n = 1 + rng() % 5000; break;
            case 1: n = 1 + rng() % (1ull << 22); break;
            case 2: n = (1ull << (10 + rng() % 22)) + (rng() % 3) - 1; break;
            case 3: n = 0xffffffffull - rng() % 4096; break;
            default: n = 1 + rng() % 0xffffffffull; break;
        }
        const uint32_t cus = cu_counts[rng() % (sizeof(cu_counts) / sizeof(cu_counts[0]))];
        const SlotPlan p = slot_plan(n, cus);
        ++cases;
        const uint64_t tiles = (n + SLOT_TILE - 1) / SLOT_TILE;
        if (p.ntiles != tiles) fail("tile count", n, cus);
        if (p.tpt < 1 || p.tpt > 63) fail("tiles per thread out of range", n, cus);
        if ((uint64_t)p.nseg * SLOT_SCAN_TILES * p.tpt < tiles) fail("second pass does not cover the tiles", n, cus);
        if (p.nseg > tiles / SLOT_SCAN_TILES + 1) fail("more workgroups than the scan state is sized for", n, cus);
        // scan state of the second pass: header, a descriptor per workgroup and per 64
        const size_t scan = 64 + 8 * ((size_t)p.nseg + ((size_t)p.nseg + 63) / 64);
        if (scan > p.counts_at) fail("scan state runs into the counts", n, cus);
        if (p.counts_at % 256 || p.place_at % 256 || p.dense_at % 256 || p.slots_at % 256) fail("misaligned part", n, cus);
        if (p.counts_at + 2 * tiles > p.place_at) fail("counts run into the places", n, cus);
        if (p.place_at + 4 * tiles > p.dense_at) fail("places run into the list", n, cus);
        if (p.dense_at + 4 * tiles > p.slots_at) fail("list runs into the slots", n, cus);
        const uint64_t groups = (tiles + SLOT_GROUP - 1) / SLOT_GROUP;
        if (p.slots_at + 8 * (uint64_t)SLOT_C * SLOT_GROUP * groups > p.bytes) fail("slots run past the end", n, cus);
        // the size a caller is told (computed for 256 compute units) holds for any device
        if (p.bytes > slot_ws_bytes(n)) fail("a device needs more than slot_ws_bytes says", n, cus);
        if (n >= RS_SAMPLE_MIN_N && refresh_ws_bytes(n) < threshold_ws_min_bytes() + refresh_scan_bytes(n) +
                                                             round_up_256(p.bytes) + 8 * (n / 16))
            fail("refresh workspace has no room for slots and n/16 candidates", n, cus);
        // the one-kernel form: a launch never has more workgroups than descriptors
        const SelectShape s = select_shape(n, cus);
        const size_t one = 64 + 8 * ((size_t)s.nseg + ((size_t)s.nseg + 63) / 64);
        if (one > select_ws_bytes(n)) fail("one-kernel scan state exceeds select_ws_bytes", n, cus);
        if ((uint64_t)s.nseg * SEL_WAVES * s.piece < n) fail("one-kernel pieces do not cover the vector", n, cus);
        if (s.piece > SEL_PIECE_MAX || s.piece % 256) fail("piece length", n, cus);
    }
    std::printf("%ld cases, %ld violations\n", cases, bad);
    return bad ? 1 : 0;
}
