// Host-side exhaustive/random check of the register sorting networks (compiled by
// tests/test_sortnet_cpu.py with hipcc for the host only; runs on the CPU).
#include <algorithm>
#include <cstdio>
#include <cstdint>
#include <random>
#include <vector>
#include "fg_sortnet.hpp"

template <int N>
static int check_sort(std::mt19937_64& rng)
{
    for (int rep = 0; rep < 2000; ++rep) {
        uint64_t v[N];
        std::vector<uint64_t> ref(N);
        for (int i = 0; i < N; ++i) { v[i] = rng() % (rep % 3 == 0 ? 7 : ~0ull); ref[i] = v[i]; }
        fg::net_sort<N>(v);
        std::sort(ref.begin(), ref.end());
        for (int i = 0; i < N; ++i) if (v[i] != ref[i]) return 1;
    }
    return 0;
}

template <int KC, int P>
static int check_absorb(std::mt19937_64& rng)
{
    for (int rep = 0; rep < 2000; ++rep) {
        uint64_t best[KC], pend[P];
        std::vector<uint64_t> all;
        for (int i = 0; i < KC; ++i) best[i] = (rep % 5 == 0 && i > KC / 2) ? ~0ull : rng() % (rep % 3 == 0 ? 9 : ~0ull);
        for (int i = 0; i < P; ++i) pend[i] = (rep % 7 == 0 && i > 2) ? ~0ull : rng() % (rep % 3 == 0 ? 9 : ~0ull);
        std::sort(best, best + KC);
        std::sort(pend, pend + P);
        all.insert(all.end(), best, best + KC);
        all.insert(all.end(), pend, pend + P);
        std::sort(all.begin(), all.end());
        fg::net_absorb<KC, P>(best, pend);
        for (int i = 0; i < KC; ++i) if (best[i] != all[i]) return 1;
    }
    return 0;
}

int main()
{
    std::mt19937_64 rng(12345);
    int bad = 0;
    bad |= check_sort<2>(rng) | check_sort<4>(rng) | check_sort<8>(rng) | check_sort<16>(rng) | check_sort<32>(rng) | check_sort<64>(rng);
    bad |= check_absorb<16, 16>(rng) | check_absorb<32, 16>(rng) | check_absorb<64, 16>(rng) | check_absorb<32, 8>(rng) |
           check_absorb<64, 32>(rng) | check_absorb<16, 8>(rng) | check_absorb<128, 16>(rng) |
           check_absorb<48, 16>(rng) | check_absorb<24, 8>(rng) | check_absorb<96, 16>(rng) | check_absorb<80, 16>(rng);
    std::printf(bad ? "FAIL\n" : "OK\n");
    return bad;
}
