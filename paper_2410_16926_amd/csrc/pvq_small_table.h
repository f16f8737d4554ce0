// Host helpers shared by the builders of the D = 8 decoder tables: N(d,k) for d <= 8 in 64 bits, the order in
// which the enumeration visits a coordinate's values, small integers as bf16.
#pragma once

#include <cstdint>
#include <cstring>
#include <vector>

namespace pvq_small {

// N(d,k) for d <= 8, small k, in 64 bits (checked against 32-bit use by the caller)
struct SmallTable {
    int K;
    std::vector<uint64_t> n;  // (9) x (K+1)
    explicit SmallTable(int K_) : K(K_), n((size_t)9 * (K_ + 1))
    {
        for (int k = 0; k <= K; k++) at(0, k) = (k == 0);
        for (int d = 1; d <= 8; d++) {
            at(d, 0) = 1;
            for (int k = 1; k <= K; k++) at(d, k) = at(d - 1, k) + at(d, k - 1) + at(d - 1, k - 1);
        }
    }
    uint64_t &at(int d, int k) { return n[(size_t)d * (K + 1) + k]; }
    uint64_t at(int d, int k) const { return n[(size_t)d * (K + 1) + k]; }
};

// coordinate values in the order the enumeration visits them: 0, +1, -1, ..., +k, -k
inline std::vector<int> visiting_order(int k)
{
    std::vector<int> v{0};
    for (int j = 1; j <= k; j++) { v.push_back(j); v.push_back(-j); }
    return v;
}

inline uint32_t bf16_of_int(int v)
{
    float f = (float)v;
    uint32_t u;
    memcpy(&u, &f, 4);
    return u >> 16;  // exact: |v| <= 256 has at most 8 significant bits
}

// the coordinate-by-coordinate walk of App. B.3 for index c of P(8,K): the yardstick of the self-tests
inline void plain_walk(const SmallTable &N, int K, uint64_t c, int (&y)[8])
{
    int k = K;
    uint64_t r = c;
    for (int i = 0; i < 7; i++) {
        const int dp = 7 - i;
        y[i] = 0;
        if (k == 0) continue;
        if (r < N.at(dp, k)) continue;
        r -= N.at(dp, k);
        int j = 1;
        while (j < k && r >= 2 * N.at(dp, k - j)) { r -= 2 * N.at(dp, k - j); j++; }
        if (r < N.at(dp, k - j)) y[i] = j; else { y[i] = -j; r -= N.at(dp, k - j); }
        k -= j;
    }
    y[7] = r == 0 ? k : -k;
}

}  // namespace pvq_small
