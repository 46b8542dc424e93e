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
    std::printf("%ld cases, %ld disagreements\n", cases, bad);
    return bad != 0;
}
