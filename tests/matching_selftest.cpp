// Host-only check of the two maximum-weight matching solvers against each other
// and against brute force: the blossom algorithm must reach the weight of the
// exact subset recursion on random graphs, and both must return valid matchings.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "matching.hpp"

static uint64_t rng_state = 88172645463325252ull;
static uint32_t rnd() {
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return uint32_t(rng_state >> 11);
}

static int64_t brute(int k, const std::vector<int64_t>& w, std::vector<char>& used, int from) {
    while (from < k && used[from]) ++from;
    if (from >= k) return 0;
    used[from] = 1;
    int64_t best = brute(k, w, used, from + 1);           // leave `from` unmatched
    for (int j = from + 1; j < k; ++j)
        if (!used[j] && w[size_t(from) * k + j] > 0) {
            used[j] = 1;
            const int64_t c = w[size_t(from) * k + j] + brute(k, w, used, from + 1);
            if (c > best) best = c;
            used[j] = 0;
        }
    used[from] = 0;
    return best;
}

static bool valid(int k, const std::vector<int64_t>& w, const std::vector<int>& mate, int64_t claimed) {
    int64_t total = 0;
    for (int a = 0; a < k; ++a) {
        const int b = mate[a];
        if (b < 0) continue;
        if (b >= k || b == a || mate[b] != a || w[size_t(a) * k + b] <= 0) return false;
        if (b > a) total += w[size_t(a) * k + b];
    }
    return total == claimed;
}

int main() {
    int trials = 0;
    for (int t = 0; t < 6000; ++t) {
        const int k = 2 + int(rnd() % 15);                  // 2 .. 16 vertices
        const int style = int(rnd() % 4);
        const int density = 20 + int(rnd() % 81);           // percent
        std::vector<int64_t> w(size_t(k) * k, 0);
        for (int a = 0; a < k; ++a)
            for (int b = a + 1; b < k; ++b) {
                if (int(rnd() % 100) >= density) continue;
                int64_t v;
                if (style == 0) v = 1 + rnd() % 3;                                   // many ties
                else if (style == 1) v = 1 + rnd() % 1000;
                else if (style == 2) v = (int64_t(1 + rnd() % 2) << 20) + rnd() % 64; // the planner's shape
                else v = 1;                                                           // maximum cardinality
                w[size_t(a) * k + b] = w[size_t(b) * k + a] = v;
            }
        std::vector<int> m1, m2;
        const int64_t exact = sar::max_weight_matching_subsets(k, w, m1);
        const int64_t bloss = sar::max_weight_matching_blossom(k, w, m2);
        if (!valid(k, w, m1, exact) || !valid(k, w, m2, bloss) || exact != bloss) {
            std::printf("mismatch: trial %d k=%d style=%d exact=%lld blossom=%lld\n", t, k, style,
                        (long long)exact, (long long)bloss);
            return 1;
        }
        if (k <= 10) {
            std::vector<char> used(k, 0);
            if (brute(k, w, used, 0) != exact) {
                std::printf("subset recursion disagrees with brute force: trial %d k=%d\n", t, k);
                return 1;
            }
        }
        ++trials;
    }
    // larger graphs: the blossom result must at least be a valid matching, twice the same
    for (int t = 0; t < 40; ++t) {
        const int k = 30 + int(rnd() % 100);
        std::vector<int64_t> w(size_t(k) * k, 0);
        for (int a = 0; a < k; ++a)
            for (int b = a + 1; b < k; ++b)
                if (rnd() % 3) w[size_t(a) * k + b] = w[size_t(b) * k + a] = (int64_t(1 + rnd() % 2) << 20) + rnd() % 200;
        std::vector<int> m;
        const int64_t got = sar::max_weight_matching_blossom(k, w, m);
        if (!valid(k, w, m, got)) {
            std::printf("invalid matching at k=%d\n", k);
            return 1;
        }
        ++trials;
    }
    std::printf("matching_selftest: %d graphs ok\n", trials);
    return 0;
}
