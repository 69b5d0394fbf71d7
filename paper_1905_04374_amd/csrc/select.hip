// Selection: Krum scores and the rounds of multi-Krum that extract theta
// gradients (Algorithm 1, function multi-Krum and the loop of multi-Bulyan).
//
// O(theta n^2) scalar work on an n x n matrix, n <= 64: one workgroup.
// Eight waves first order every row of the distance matrix once (rank by
// counting, keys (distance, index)); then a single wave, lane i = gradient i,
// plays the rounds with a bit mask of the ranks of its ordered row that are still
// active: the first score is the sum of the q nearest distances in ascending order
// in fp64, later ones follow by one subtraction per round; find the smallest
// (score, index) by a wave reduction, extract it.  When the
// averaged sets are wanted every score has to be ranked in every round: the
// scores go through LDS and all eight waves count, each over an eighth of the
// gradients.
#include <hip/hip_runtime.h>

#include "alg1_plan.hpp"
#include "gram_combine.hpp"
#include "mb_internal.hpp"

namespace mb {
namespace {

constexpr int kSelThreads = 512;   // 8 waves rank the rows, two per SIMD: each may still use 256 registers
constexpr int kPerThread = kMaxN * kMaxN / kSelThreads;

struct Rounds {
    const double *sD;            // LDS: row i in ascending order
    const unsigned char *sJ;     // LDS: neighbour index by rank within row i
    const unsigned char *sR;     // LDS: rank of neighbour j within row i
    int n, f, rounds;
    const uint8_t *active_in;
    int32_t *sel;
    uint8_t *agr_sets;
    int32_t *m_out;
    double *scores_out;
    double *sS;                  // LDS, 64 scores of the current round      } only when the sets are
    unsigned long long *sAct;    // LDS, the active gradients of that round  } wanted: see
    unsigned char *sCnt;         // LDS, [lane][wave] partial counts         } count_before
};

__device__ __forceinline__ double read_lane(double x, int lane)   // lane: the same for the whole wave
{
    const unsigned long long u = (unsigned long long)__double_as_longlong(x);
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)u, lane);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(u >> 32), lane);
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

template <int CTRL>
__device__ __forceinline__ double dpp_move(double x)   // x of the lane the DPP control selects
{
    const unsigned long long u = (unsigned long long)__double_as_longlong(x);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(unsigned)u, CTRL, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(unsigned)(u >> 32), CTRL, 0xf, 0xf, true);
    return __longlong_as_double((long long)(((unsigned long long)(unsigned)hi << 32) | (unsigned)lo));
}

constexpr int kSelWaves = kSelThreads / 64;

// Wave `wave` of kSelWaves, lane i: how many active gradients j = wave, wave + 8, ... come before
// gradient i in the order (score, index).  Scores of lanes that hold no active gradient are +inf
// and their bit in `act` is clear.
__device__ __forceinline__ void count_before(const double *sS, unsigned long long act, int wave, int i,
                                             unsigned char *sCnt)
{
    const double S = sS[i];
    double Sj[64 / kSelWaves];
#pragma unroll
    for (int k = 0; k < 64 / kSelWaves; ++k) Sj[k] = sS[wave + kSelWaves * k];
    int cnt = 0;
#pragma unroll
    for (int k = 0; k < 64 / kSelWaves; ++k) {
        const int j = wave + kSelWaves * k;
        if ((act >> j) & 1ull) cnt += (Sj[k] < S || (Sj[k] == S && j < i)) ? 1 : 0;
    }
    sCnt[i * kSelWaves + wave] = (unsigned char)cnt;
}

// The waves that do not play the rounds: one count per round, between the two barriers of that
// round (the same two that play_rounds goes through).
__device__ __forceinline__ void help_rounds(const Rounds &a, int wave, int i)
{
    for (int t = 0; t < a.rounds; ++t) {
        __syncthreads();
        count_before(a.sS, *a.sAct, wave, i, a.sCnt);
        __syncthreads();
    }
}

// Sum of the distances of one ordered row at the ranks set in `take`, added in ascending order.
__device__ __forceinline__ double sum_taken(const double *rowD, unsigned long long take)
{
    double S = 0.0;
    while (take) {
        const int r = (int)__builtin_ctzll(take);
        take &= take - 1ull;
        S += rowD[r];
    }
    return S;
}

// One wave, lane i = gradient i, its ordered row in LDS.
// `near`: bit r set while the r-th nearest neighbour of i is still active.
// `take`: the q lowest set bits of `near`, the neighbours whose distances make up the score.
// From one round to the next q drops by one and at most one neighbour leaves, so `take` loses
// either the bit of the extracted gradient or its own top bit: no search after the first round,
// and the score follows by one subtraction.  The first round's scores are the plain sums in
// ascending order.  Later ones carry the rounding of the subtractions (a few 1e-16 of the score),
// except where exact ties live: a score of one distance (two gradients that are each other's last
// neighbour hold the same one) is that distance, and copies of a gradient go through identical
// operations on identical values.  A row with infinite distances is summed afresh (no inf - inf).
__device__ __forceinline__ void play_rounds(const Rounds &a, int i)
{
    const int n = a.n, f = a.f;
    const double inf = __builtin_huge_val();
    const int row = i < n ? i : 0;
    const double *rowD = a.sD + row * kMaxN;

    unsigned long long act = 0;   // active gradients, same value in every lane
    for (int j = 0; j < n; ++j)
        if (!a.active_in || a.active_in[j]) act |= 1ull << j;
    unsigned long long near = n >= 2 ? (~0ull >> (65 - n)) : 0ull;   // all n - 1 neighbours
    if (a.active_in) {
        near = 0;
        for (int r0 = 0; r0 < n - 1; r0 += 8) {
            int jn[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) jn[q] = a.sJ[row * kMaxN + ((r0 + q) & (kMaxN - 1))];
#pragma unroll
            for (int q = 0; q < 8; ++q)
                if (r0 + q < n - 1 && ((act >> jn[q]) & 1ull)) near |= 1ull << (r0 + q);
        }
    }
    unsigned long long take = 0;
    {
        int q = __popcll(act) - f - 2;
        q = q < 0 ? 0 : q;
        int lo = 0, hi = 64;                       // smallest cut with popc(near & below(cut)) >= q
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            const unsigned long long below = mid >= 64 ? ~0ull : ((1ull << mid) - 1ull);
            if ((int)__popcll(near & below) >= q) hi = mid; else lo = mid + 1;
        }
        take = near & (lo >= 64 ? ~0ull : ((1ull << lo) - 1ull));
    }
    double sum = 0.0;   // over `take`, ascending; eight reads in flight
    for (int r0 = 0; r0 < n - 1; r0 += 8) {
        double u[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) u[q] = rowD[(r0 + q) & (kMaxN - 1)];
#pragma unroll
        for (int q = 0; q < 8; ++q)
            if ((take >> (r0 + q)) & 1ull) sum += u[q];
    }

    for (int t = 0; t < a.rounds; ++t) {
        const int k = __popcll(act);
        int q = k - f - 2;
        q = q < 0 ? 0 : q;
        const bool mine = i < n && ((act >> i) & 1ull);
        const double S = mine ? sum : inf;
        if (t == 0 && a.scores_out && i < n) a.scores_out[i] = S;

        int w;            // the first of the active gradients in the order (score, index)
        if (a.agr_sets) {
            // position of i in that order: every wave counts over its eighth of the gradients
            a.sS[i] = S;
            if (i == 0) *a.sAct = act;
            __syncthreads();
            count_before(a.sS, act, 0, i, a.sCnt);
            __syncthreads();
            const uint2 c = *reinterpret_cast<const uint2 *>(a.sCnt + i * kSelWaves);   // 8 counts of at most 8
            const int pos = (int)((c.x * 0x01010101u) >> 24) + (int)((c.y * 0x01010101u) >> 24);
            const unsigned long long first = __ballot(mine && pos == 0);
            w = first ? (int)__builtin_ctzll(first) : 0;
            if (i < n) a.agr_sets[t * n + i] = (mine && pos < q) ? 1 : 0;
        } else {
            // smallest score of the wave, then the first active lane that has it: the same as
            // the smallest (score, index).  Data-parallel moves inside rows of 16 lanes (min is
            // idempotent, so swaps and mirrors do), lane reads across the four rows.
            double mn = S;
            mn = fmin(mn, dpp_move<0xB1>(mn));     // quad_perm [1,0,3,2]
            mn = fmin(mn, dpp_move<0x4E>(mn));     // quad_perm [2,3,0,1]
            mn = fmin(mn, dpp_move<0x141>(mn));    // row_half_mirror
            mn = fmin(mn, dpp_move<0x140>(mn));    // row_mirror
            const double best = fmin(fmin(read_lane(mn, 0), read_lane(mn, 16)),
                                     fmin(read_lane(mn, 32), read_lane(mn, 48)));
            const unsigned long long first = __ballot(mine && S == best);
            w = first ? (int)__builtin_ctzll(first) : 0;
        }
        if (a.sel && i == 0) a.sel[t] = w;
        if (a.m_out && i == 0) a.m_out[t] = q < k ? q : k;
        if (k > 0) {
            act &= ~(1ull << w);
            const int rw = a.sR[row * kMaxN + w];        // rank of the extracted gradient in row i
            const unsigned long long wbit = (w != row) ? (1ull << rw) : 0ull;
            near &= ~wbit;
            int qn = k - 1 - f - 2;
            qn = qn < 0 ? 0 : qn;
            if (qn < q && take) {
                const int gone = (take & wbit) ? rw : 63 - (int)__builtin_clzll(take);
                take &= ~(1ull << gone);
                const double x = rowD[gone];
                if ((take & (take - 1ull)) == 0ull || !(x < inf)) sum = sum_taken(rowD, take);
                else sum -= x;
            }
        }
    }
}

// dist != null: the distance matrix.  Otherwise gram (and gram2, gate: the second pass, if one was
// launched) = the reduced Gram tiles of the distance pass, and the matrix is formed here exactly as
// finalize_gram_kernel forms it.
// plan != null (needs sel and agr_sets): the plan of the Algorithm-1 coordinate pass for the
// chosen gradients and sets is written as well, once the last round is over.
__global__ __launch_bounds__(kSelThreads) void select_kernel(
    const double *__restrict__ dist, const double *__restrict__ gram, const double *__restrict__ gram2,
    const int *__restrict__ gate, int n, int f, int rounds,
    const uint8_t *__restrict__ active_in, int32_t *__restrict__ sel, uint8_t *__restrict__ agr_sets,
    int32_t *__restrict__ m_out, double *__restrict__ scores_out, int32_t *__restrict__ plan,
    const double *__restrict__ prep_ordered, const unsigned char *__restrict__ prep_idx)
{
    __shared__ double sD[kMaxN * kMaxN];        // first dist[i][j], then row i in ascending order
    __shared__ unsigned char sJ[kMaxN * kMaxN]; // neighbour index by rank within row i
    __shared__ unsigned char sR[kMaxN * kMaxN]; // rank of neighbour j within row i
    __shared__ int rep[kMaxN];
    __shared__ double sS[64];
    __shared__ unsigned long long sAct;
    __shared__ __attribute__((aligned(8))) unsigned char sCnt[64 * kSelWaves];
    static_assert(kSelWaves == 8 && kMaxN <= 64, "count_before: eight counts of at most eight per lane");
    const int tid = threadIdx.x;
    const double inf = __builtin_huge_val();

    // the ordered rows as the second distance pass has left them (it had nothing else to do)
    const bool prepared = !dist && prep_ordered && gate && gate[kGateFlag] == 0;
    if (prepared) {
        double x[kPerThread];
        unsigned char bj[kPerThread], br[kPerThread];
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            const int e = tid + k * kSelThreads;         // entry (row e / 64, column e % 64) of the padded arrays
            const bool in = (e >> 6) < n && (e & 63) < n;
            x[k] = in ? prep_ordered[e] : 0.0;
            bj[k] = in ? prep_idx[e] : 0;
            br[k] = in ? prep_idx[kMaxN * kMaxN + e] : 0;
        }
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            const int e = tid + k * kSelThreads;
            sD[e] = x[k];
            sJ[e] = bj[k];
            sR[e] = br[k];
        }
        __syncthreads();
    } else if (dist) {
        double x[kPerThread];
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            const int e = tid + k * kSelThreads;
            x[k] = e < n * n ? dist[e] : 0.0;
        }
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            const int e = tid + k * kSelThreads;
            if (e < n * n) sD[(e / n) * kMaxN + (e % n)] = (x[k] == x[k]) ? x[k] : inf;   // a NaN distance never makes a neighbour
        }
        __syncthreads();
    } else {
        // which rows are copies of an earlier row (their Gram entries are bit-identical), then every
        // pair from the pass with the smaller error bound; the Gram entries of all of a thread's
        // elements first (many loads in flight), the arithmetic after
        const bool refined = gate && gate[kGateFlag] != 0;
        if (tid < kMaxN) rep[tid] = tid;
        __syncthreads();
        bool same[kPerThread];
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            const int e = tid + k * kSelThreads;
            same[k] = false;
            if (e < n * n && e / n > e % n) same[k] = gram_term(gram, e / n, e % n).same;
        }
#pragma unroll
        for (int k = 0; k < kPerThread; ++k)
            if (same[k]) atomicMin(&rep[(tid + k * kSelThreads) / n], (tid + k * kSelThreads) % n);
        __syncthreads();
        double mine[kPerThread];
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            const int e = tid + k * kSelThreads;
            mine[k] = 0.0;
            if (e < n * n) {
                const int i = rep[e / n], j = rep[e % n];
                if (i != j) mine[k] = gram_pair_distance(gram, gram2, refined, i > j ? i : j, i > j ? j : i);
            }
        }
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            const int e = tid + k * kSelThreads;
            if (e < n * n) {
                double x = mine[k];
                if (!(x == x)) x = inf;
                sD[(e / n) * kMaxN + (e % n)] = x;
            }
        }
        __syncthreads();
    }

    if (!prepared) {
        // rank of j among the neighbours of i (everything but i itself), keys (distance, index)
        double myv[kPerThread];
        int myrank[kPerThread];
    #pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            const int e = tid + k * kSelThreads;
            myrank[k] = -1;
            myv[k] = 0.0;
            if (e < n * n) {
                const int i = e / n, j = e % n;
                if (i != j) {
                    const double v = sD[i * kMaxN + j];
                    int rank = 0;
                    // one wave per SIMD, nothing else hides the LDS latency: eight reads in flight
                    // (entries past n in the padded row are never counted)
                    for (int j0 = 0; j0 < n; j0 += 8) {
                        double u[8];
    #pragma unroll
                        for (int q = 0; q < 8; ++q) u[q] = sD[i * kMaxN + ((j0 + q) & (kMaxN - 1))];
    #pragma unroll
                        for (int q = 0; q < 8; ++q) {
                            const int jj = j0 + q;
                            rank += (jj < n && jj != i && (u[q] < v || (u[q] == v && jj < j))) ? 1 : 0;
                        }
                    }
                    myrank[k] = rank;
                    myv[k] = v;
                }
            }
        }
        __syncthreads();
    #pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            const int e = tid + k * kSelThreads;
            if (myrank[k] >= 0) {
                const int i = e / n, j = e % n;
                sD[i * kMaxN + myrank[k]] = myv[k];
                sJ[i * kMaxN + myrank[k]] = (unsigned char)j;
                sR[i * kMaxN + j] = (unsigned char)myrank[k];
            }
        }
        __syncthreads();
    }
    const Rounds rd{sD, sJ, sR, n, f, rounds, active_in, sel, agr_sets, m_out, scores_out, sS, &sAct, sCnt};
    if (tid >= 64) {   // one wave plays the rounds; the others only help to rank the scores for the sets
        if (agr_sets) help_rounds(rd, tid >> 6, tid & 63);
    } else {
        play_rounds(rd, tid);
    }
    if (!plan) return;
    __syncthreads();   // sel and agr_sets as the first wave has written them
    alg1_plan_body<kSelThreads>(n, rounds, sel, agr_sets, plan, tid);
}

}  // namespace

hipError_t launch_select(const double *dist, int n, int f, int rounds, const uint8_t *active_in,
                         int32_t *sel, uint8_t *agr_sets, int32_t *m_out, double *scores_out, int32_t *plan,
                         hipStream_t s)
{
    if (plan && !(sel && agr_sets)) return hipErrorInvalidValue;
    select_kernel<<<dim3(1), dim3(kSelThreads), 0, s>>>(dist, nullptr, nullptr, nullptr, n, f, rounds, active_in, sel,
                                                        agr_sets, m_out, scores_out, plan, nullptr, nullptr);
    return hipGetLastError();
}

hipError_t launch_select_gram(const double *reduced, const double *reduced2, const int *gate, int n, int f,
                              int rounds, int32_t *sel, uint8_t *agr_sets, int32_t *m_out, int32_t *plan,
                              const double *prep_ordered, const unsigned char *prep_idx, hipStream_t s)
{
    if (plan && !(sel && agr_sets)) return hipErrorInvalidValue;
    select_kernel<<<dim3(1), dim3(kSelThreads), 0, s>>>(nullptr, reduced, reduced2, gate, n, f, rounds, nullptr, sel,
                                                        agr_sets, m_out, nullptr, plan, prep_ordered, prep_idx);
    return hipGetLastError();
}

}  // namespace mb
