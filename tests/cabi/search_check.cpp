// Host check of the index searches the reduce's boundary kernels use: against
// std::lower_bound on random sorted lists (with and without duplicates, narrow
// and wide value ranges), over random sub-ranges, with guesses anywhere from far
// before the range to far behind it.  Prints the number of cases and exits 0,
// or prints the first disagreements and exits 1.
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <random>
#include <vector>

#include "okt_search.h"

int main() {
    std::mt19937_64 rng(20220117);
    long bad = 0, cases = 0;
    for (int rep = 0; rep < 300000; ++rep) {
        int n = (int)(rng() % 300);
        const uint32_t span = rng() % 3 == 0 ? 40u : rng() % 3 == 0 ? 0xffffffffu : 100000u;
        std::vector<uint32_t> v(n);
        for (auto& x : v) x = (uint32_t)(rng() % span);
        std::sort(v.begin(), v.end());
        if (rng() % 2) v.erase(std::unique(v.begin(), v.end()), v.end());
        n = (int)v.size();
        const uint64_t lo = n ? rng() % (n + 1) : 0, hi = n ? lo + rng() % (n - lo + 1) : 0;
        const uint32_t x = rng() % 4 == 0 && n ? v[rng() % n] : (uint32_t)(rng() % span) + (uint32_t)(rng() % 3);
        const uint64_t guess = rng() % (uint64_t)(n + 40);
        const uint64_t want = (uint64_t)(std::lower_bound(v.begin() + lo, v.begin() + hi, x) - v.begin());
        const uint64_t a = okt::lower_bound_idx(v.data(), lo, hi, x);
        const uint64_t b = okt::lower_bound_near(v.data(), lo, hi, x, guess);
        ++cases;
        if (a != want || b != want) {
            if (bad < 5)
                std::printf("n=%d lo=%llu hi=%llu x=%u guess=%llu: want %llu, bisection %llu, from guess %llu\n",
                            n, (unsigned long long)lo, (unsigned long long)hi, x, (unsigned long long)guess,
                            (unsigned long long)want, (unsigned long long)a, (unsigned long long)b);
            ++bad;
        }
    }
    // the balanced split (okt_region_partition): quantile positions of the sorted
    // list and where each region begins, against the rule written out with
    // std::lower_bound; and a count no select can produce (above n), which must be
    // answered without a single read of the list
    for (int rep = 0; rep < 20000; ++rep) {
        const uint64_t n = 1 + rng() % 5000;
        const uint32_t R = 1 + (uint32_t)(rng() % 70);
        std::vector<uint32_t> v;
        const int kind = (int)(rng() % 4);             // empty, sparse, clustered low, dense
        const uint64_t want_nnz = kind == 0 ? 0 : kind == 3 ? n : 1 + rng() % n;
        for (uint64_t i = 0; i < n && v.size() < want_nnz; ++i)
            if (kind == 3 || kind == 2 || rng() % n < want_nnz) v.push_back((uint32_t)i);
        const uint64_t nnz = v.size();
        for (uint64_t r = 0; r <= R; ++r) {
            uint32_t wb;
            uint64_t wo;
            if (r == 0) { wb = 0; wo = 0; }
            else if (r == R) { wb = (uint32_t)n; wo = nnz; }
            else if (nnz == 0) { wb = (uint32_t)(r * n / R); wo = 0; }
            else {
                wb = v[(size_t)(r * nnz / R)];
                wo = (uint64_t)(std::lower_bound(v.begin(), v.end(), wb) - v.begin());
            }
            const okt::PartitionCut c = okt::partition_cut(v.data(), nnz, n, R, r);
            ++cases;
            if (c.bound != wb || c.offset != wo) {
                if (bad < 5) std::printf("partition n=%llu R=%u r=%llu nnz=%llu: want (%u, %llu), got (%u, %llu)\n",
                                         (unsigned long long)n, R, (unsigned long long)r, (unsigned long long)nnz, wb,
                                         (unsigned long long)wo, c.bound, (unsigned long long)c.offset);
                ++bad;
            }
            // the failure word: idx is a null pointer here, any read of it would crash
            const okt::PartitionCut f = okt::partition_cut(nullptr, ~0ull, n, R, r);
            const uint32_t fb = r == R ? (uint32_t)n : (uint32_t)(r * n / R);
            ++cases;
            if (f.bound != fb || f.offset != ~0ull) {
                if (bad < 5) std::printf("partition of a failed count: r=%llu got (%u, %llu)\n",
                                         (unsigned long long)r, f.bound, (unsigned long long)f.offset);
                ++bad;
            }
        }
    }
    std::printf("%ld cases, %ld disagreements\n", cases, bad);
    return bad != 0;
}
