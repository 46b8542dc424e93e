// Searches in a sorted index list, written so that a host compiler can build them
// too (the CPU tests check them against std::lower_bound).
#ifndef OKT_SEARCH_H
#define OKT_SEARCH_H

#include <stdint.h>

#ifdef __HIPCC__
#define OKT_SEARCH_FN __host__ __device__ __forceinline__
#else
#define OKT_SEARCH_FN static inline
#endif

namespace okt {

// The first position in [lo, hi) whose entry is not below x, or hi.
OKT_SEARCH_FN uint64_t lower_bound_idx(const uint32_t* a, uint64_t lo, uint64_t hi, uint32_t x) {
    while (lo < hi) {
        const uint64_t mid = lo + ((hi - lo) >> 1);
        if (a[mid] < x) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// The same answer - the first position in [lo, hi) whose entry is not below x, or
// hi - found from a guess: one probe at the guess, then steps of doubling length
// away from it until x is bracketed, then the bisection inside the bracket.  With
// indices spread evenly over the region the guess is a few dozen entries off, so
// a boundary costs about half the probes of a bisection over the whole list, all
// but the first in two or three neighbouring cache lines; with any other spread
// it costs at most about twice the bisection.
OKT_SEARCH_FN uint64_t lower_bound_near(const uint32_t* a, uint64_t lo, uint64_t hi, uint32_t x,
                                        uint64_t guess) {
    if (lo >= hi) return lo;
    uint64_t g = guess < lo ? lo : (guess >= hi ? hi - 1 : guess);
    uint64_t step = 16;
    if (a[g] < x) {                              // the answer lies in (g, hi]
        uint64_t first = g + 1;
        for (;;) {
            const uint64_t p = g + step;
            if (p >= hi) return lower_bound_idx(a, first, hi, x);
            if (!(a[p] < x)) return lower_bound_idx(a, first, p, x);
            first = p + 1;
            g = p;
            step *= 2;
        }
    }
    uint64_t last = g;                           // a[last] is not below x: the answer lies in [lo, last]
    for (;;) {
        if (last - lo < step) return lower_bound_idx(a, lo, last, x);
        const uint64_t p = last - step;
        if (a[p] < x) return lower_bound_idx(a, p + 1, last, x);
        last = p;
        step *= 2;
    }
}

// Boundary r (0 <= r <= R) of the balanced split of [0, n) by a sorted index list
// of nnz entries (Sec. 3.1.1), and the list position where region r begins:
// b[r] = idx[floor(r * nnz / R)], b[0] = 0, b[R] = n; without entries the equal
// split floor(r * n / R).  A count above n cannot come from a select over n
// elements - it is the all-ones word a failed call leaves in its counts - and is
// answered without reading idx: the equal split, every offset all ones, so that
// whatever consumes the offsets sees empty slices and the failure stays visible.
struct PartitionCut { uint32_t bound; uint64_t offset; };
OKT_SEARCH_FN PartitionCut partition_cut(const uint32_t* idx, uint64_t nnz, uint64_t n, uint32_t R,
                                         uint64_t r) {
    if (nnz > n) return PartitionCut{r == R ? (uint32_t)n : (uint32_t)((r * n) / R), ~0ull};
    if (r == 0) return PartitionCut{0u, 0ull};
    if (r == R) return PartitionCut{(uint32_t)n, nnz};
    if (nnz == 0) return PartitionCut{(uint32_t)((r * n) / R), 0ull};     // r, n < 2^32: no overflow
    const uint32_t b = idx[(r * nnz) / R];                                 // r, nnz < 2^32
    return PartitionCut{b, lower_bound_idx(idx, 0, nnz, b)};
}

}  // namespace okt
#endif
