// Host-side check of the comparator networks the coordinate kernels apply in registers (built and run
// by tests/test_sortnet_host.py; no GPU involved: the functions are __host__ __device__).
// For every N = 1..64: the zero-one principle (a network sorts every input iff it sorts every 0/1
// input) exhaustively up to N = 14 and on 20 000 random 0/1 inputs beyond, plus random float keys
// with repeats against std::sort; the packed 16-bit and the 64-bit comparators on random keys.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <random>

#include "../paper_1905_04374_amd/csrc/sortnet.hpp"

static std::mt19937_64 rng(1905);

template <int N>
static bool check()
{
    float v[N], w[N];
    const uint64_t exhaustive = N <= 14 ? (1ull << N) : 0;
    const uint64_t cases = exhaustive ? exhaustive : 20000;
    for (uint64_t c = 0; c < cases; ++c) {
        const uint64_t bits = exhaustive ? c : rng();
        int ones = 0;
        for (int i = 0; i < N; ++i) {
            v[i] = (float)((bits >> i) & 1);
            ones += (int)((bits >> i) & 1);
        }
        mb::sort_registers<N>(v);
        for (int i = 0; i < N; ++i)
            if (v[i] != (i >= N - ones ? 1.0f : 0.0f)) return false;
    }
    std::uniform_int_distribution<int> pick(-20, 20);
    for (int c = 0; c < 500; ++c) {
        for (int i = 0; i < N; ++i) v[i] = w[i] = 0.25f * (float)pick(rng);
        mb::sort_registers<N>(v);
        std::sort(w, w + N);
        for (int i = 0; i < N; ++i)
            if (v[i] != w[i]) return false;
    }
    // two 16-bit integer keys per word, sorted side by side; 64-bit keys
    mb::short2v p[N];
    short lo[N], hi[N];
    unsigned long long k[N], ks[N];
    for (int c = 0; c < 500; ++c) {
        for (int i = 0; i < N; ++i) {
            lo[i] = (short)rng();
            hi[i] = (short)rng();
            p[i] = mb::short2v{lo[i], hi[i]};
            k[i] = ks[i] = rng() >> (c & 1 ? 0 : 40);
        }
        mb::sort_registers<N>(p);
        mb::sort_registers<N>(k);
        std::sort(lo, lo + N);
        std::sort(hi, hi + N);
        std::sort(ks, ks + N);
        for (int i = 0; i < N; ++i)
            if (p[i][0] != lo[i] || p[i][1] != hi[i] || k[i] != ks[i]) return false;
    }
    return true;
}

template <int N>
static int check_up_to()
{
    if constexpr (N == 0) {
        return 0;
    } else {
        const int bad = check_up_to<N - 1>();
        if (!check<N>()) {
            std::printf("network for N = %d fails\n", N);
            return bad + 1;
        }
        return bad;
    }
}

int main()
{
    const int bad = check_up_to<64>();
    std::printf("%d of 64 networks fail\n", bad);
    return bad ? 1 : 0;
}
