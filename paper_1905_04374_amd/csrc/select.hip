// Selection: Krum scores and the rounds of multi-Krum that extract theta
// gradients (Algorithm 1, function multi-Krum and the loop of multi-Bulyan).
//
// O(theta n^2) scalar work on an n x n matrix, n <= 64: one workgroup.
// All 16 waves first order every row of the distance matrix once (rank by
// counting, keys (distance, index)); then a single wave, lane i = gradient i,
// plays the rounds: walk the own ordered row skipping extracted gradients,
// add the q nearest distances in ascending order in fp64, rank the scores by
// (score, index) with wave shuffles, extract the first.
#include <hip/hip_runtime.h>

#include "mb_internal.hpp"

namespace mb {
namespace {

constexpr int kSelThreads = 1024;

__global__ __launch_bounds__(kSelThreads) void select_kernel(
    const double *__restrict__ dist, int n, int f, int rounds, const uint8_t *__restrict__ active_in,
    int32_t *__restrict__ sel, uint8_t *__restrict__ agr_sets, int32_t *__restrict__ m_out,
    double *__restrict__ scores_out)
{
    __shared__ double sD[kMaxN * kMaxN];        // first dist[i][j], then row i in ascending order
    __shared__ unsigned char sJ[kMaxN * kMaxN]; // neighbour index by rank within row i
    const int tid = threadIdx.x;
    const double inf = __builtin_huge_val();

    for (int e = tid; e < n * n; e += kSelThreads) {
        double x = dist[e];
        if (!(x == x)) x = inf;                 // a NaN distance never makes a neighbour
        sD[(e / n) * kMaxN + (e % n)] = x;
    }
    __syncthreads();

    // rank of j among the neighbours of i (everything but i itself), keys (distance, index)
    double myv[4];
    int myrank[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int e = tid + k * kSelThreads;
        myrank[k] = -1;
        myv[k] = 0.0;
        if (e < n * n) {
            const int i = e / n, j = e % n;
            if (i != j) {
                const double v = sD[i * kMaxN + j];
                int rank = 0;
                for (int jj = 0; jj < n; ++jj) {
                    const double u = sD[i * kMaxN + jj];
                    rank += (jj != i && (u < v || (u == v && jj < j))) ? 1 : 0;
                }
                myrank[k] = rank;
                myv[k] = v;
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int e = tid + k * kSelThreads;
        if (myrank[k] >= 0) {
            const int i = e / n, j = e % n;
            sD[i * kMaxN + myrank[k]] = myv[k];
            sJ[i * kMaxN + myrank[k]] = (unsigned char)j;
        }
    }
    __syncthreads();
    if (tid >= 64) return;   // no barrier below this line

    const int i = tid;
    unsigned long long act = 0;   // same value in every lane
    for (int j = 0; j < n; ++j)
        if (!active_in || active_in[j]) act |= 1ull << j;

    for (int t = 0; t < rounds; ++t) {
        const int k = __popcll(act);
        int q = k - f - 2;
        q = q < 0 ? 0 : q;
        const bool mine = i < n && ((act >> i) & 1ull);
        double S = inf;
        if (mine) {
            S = 0.0;
            int cnt = 0;
            for (int r = 0; r < n - 1 && cnt < q; ++r) {
                const int j = sJ[i * kMaxN + r];
                if ((act >> j) & 1ull) {
                    S += sD[i * kMaxN + r];
                    ++cnt;
                }
            }
        }
        if (t == 0 && scores_out && i < n) scores_out[i] = S;
        // position of i in the order (score, index) of the active gradients
        int pos = 0;
        for (int j = 0; j < n; ++j) {
            const double Sj = __shfl(S, j, 64);
            const bool aj = (act >> j) & 1ull;
            pos += (aj && (Sj < S || (Sj == S && j < i))) ? 1 : 0;
        }
        const unsigned long long first = __ballot(mine && pos == 0);
        const int w = first ? (int)__builtin_ctzll(first) : 0;
        if (sel && i == 0) sel[t] = w;
        if (agr_sets && i < n) agr_sets[t * n + i] = (mine && pos < q) ? 1 : 0;
        if (m_out && i == 0) m_out[t] = q < k ? q : k;
        if (first) act &= ~(1ull << w);
    }
}

}  // namespace

hipError_t launch_select(const double *dist, int n, int f, int rounds, const uint8_t *active_in,
                         int32_t *sel, uint8_t *agr_sets, int32_t *m_out, double *scores_out,
                         hipStream_t s)
{
    select_kernel<<<dim3(1), dim3(kSelThreads), 0, s>>>(dist, n, f, rounds, active_in, sel, agr_sets,
                                                        m_out, scores_out);
    return hipGetLastError();
}

}  // namespace mb
