// Coordinate-wise phase of multi-Bulyan exactly as Algorithm 1 prints it:
// M[c] = median over t of G^ext[t][c]; G^agr[t][c] = average of the gradients
// that round t of multi-Krum averaged; out[c] = average of the beta values
// G^agr[.][c] closest to M[c].
//
// G^agr is never materialised.  In the regular case a round's set is the
// previous one minus its winner; the averages are then running sums over the
// winners' values (needed for the median anyway) on top of the last round's
// set: theta + f row streams, all in registers.  Otherwise (the order of the
// scores changed between rounds) each workgroup turns the theta x n membership
// matrix into a list of signed row updates (rows entering or leaving the set
// from one round to the next); the running sum S_t = S_{t-1} +- few rows then
// costs a handful of adds per round.  A wave stages the values of the rows it
// needs for its 64 coordinates in LDS (row-major, lane = coordinate), because
// the update lists index rows at run time.  Rows that no round uses are not
// read at all.
//
// Compiled once per group of 8 values of theta (-DMB_GROUP=0..7).
#include <hip/hip_runtime.h>

#include "mb_internal.hpp"
#include "sortnet.hpp"

#ifndef MB_GROUP
#error "compile with -DMB_GROUP=0..7"
#endif

namespace mb {
namespace {

constexpr int kThreads = 128;   // 2 waves: the staging area is n x 256 bytes per wave
constexpr int kWaves = kThreads / 64;
typedef float floatx2 __attribute__((ext_vector_type(2)));

// average of the beta values a[.] closest to med (closeness |a - med| in fp32, ties to the smaller value)
template <int THETA>
__device__ __forceinline__ float pick_closest(float (&a)[THETA], float med, int beta)
{
    if (beta == 1) {
        float best = a[0], bd = fabsf(a[0] - med);
#pragma unroll
        for (int t = 1; t < THETA; ++t) {
            const float dt = fabsf(a[t] - med);
            const bool take = dt < bd || (dt == bd && a[t] < best);
            best = take ? a[t] : best;
            bd = take ? dt : bd;
        }
        return best;
    }
    sort_registers<THETA>(a);
    float dlt[THETA];
#pragma unroll
    for (int p = 0; p < THETA; ++p) dlt[p] = fabsf(a[p] - med);
    float sum = 0.0f;
#pragma unroll
    for (int p = 0; p < THETA; ++p) {
        int rank = 0;
#pragma unroll
        for (int o = 0; o < THETA; ++o) {
            if (o < p) rank += (dlt[o] <= dlt[p]) ? 1 : 0;
            if (o > p) rank += (dlt[o] < dlt[p]) ? 1 : 0;
        }
        sum += (rank < beta) ? a[p] : 0.0f;
    }
    return sum / (float)beta;
}

// The regular case: from one round to the next the set only loses its winner, so
// set_t = set_{theta-1} + {winner_t .. winner_{theta-2}}.  The averages are then running sums over
// the winners' values, which the median needs anyway: theta + f coalesced row streams, everything
// in registers, no LDS.  The plan (winners, base rows, weights) comes from launch_alg1_plan through
// scalar loads; every workgroup takes one tile and ends (measured faster than workgroups that
// loop over tiles, as in the other coordinate kernel).  B1: beta = 1, the one average closest to
// the median is picked while the running sums are formed (half the registers); a lane then owns
// two neighbouring coordinates.
constexpr int kRegThreads = 256;
constexpr int kBaseRegs = 16;   // base rows loaded in one batch (the default theta leaves f <= 15)

template <int THETA, bool B1>
__global__ __launch_bounds__(kRegThreads) void coord_alg1_regular_kernel(
    const float *__restrict__ G, int64_t d, int64_t ld, int beta, const int32_t *__restrict__ plan,
    float *__restrict__ out)
{
    if (!plan[kPlanRegular]) return;
    constexpr int VEC = B1 ? 2 : 1;
    const int64_t c = ((int64_t)blockIdx.x * kRegThreads + threadIdx.x) * VEC;
    if (c >= d) return;
    const int nb = plan[kPlanNBase];
    const float *inv_m = reinterpret_cast<const float *>(plan + kPlanInvM);
    const bool pairs_ok = VEC == 2 && ((uintptr_t)G % 8 == 0) && (ld % 2 == 0) && ((uintptr_t)out % 8 == 0);
    const bool two = VEC == 2 && c + 1 < d;
    const bool vec = pairs_ok && two;
    float x[2];
    auto load = [&](int row) {
        const float *p = G + (int64_t)row * ld + c;
        if (vec) {
            const floatx2 v = __builtin_nontemporal_load(reinterpret_cast<const floatx2 *>(p));
            x[0] = v[0];
            x[1] = v[1];
        } else {
            x[0] = __builtin_nontemporal_load(p);
            x[1] = two ? __builtin_nontemporal_load(p + 1) : x[0];
        }
    };
    float e[VEC][THETA];
#pragma unroll
    for (int t = 0; t < THETA; ++t) {
        load(plan[kPlanWinner + t]);
#pragma unroll
        for (int k = 0; k < VEC; ++k) e[k][t] = x[k];
    }
    float S[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) S[k] = 0.0f;
    {
        float xb[VEC][kBaseRegs];
#pragma unroll
        for (int j = 0; j < kBaseRegs; ++j) {
#pragma unroll
            for (int k = 0; k < VEC; ++k) xb[k][j] = 0.0f;
            if (j < nb) {                    // same for every lane
                load(plan[kPlanBase + j]);
#pragma unroll
                for (int k = 0; k < VEC; ++k) xb[k][j] = x[k];
            }
        }
#pragma unroll
        for (int j = 0; j < kBaseRegs; ++j)
#pragma unroll
            for (int k = 0; k < VEC; ++k) S[k] += xb[k][j];
    }
    for (int s0 = kBaseRegs; s0 < nb; s0 += 8) {   // more base rows than one batch
        float xb[VEC][8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
#pragma unroll
            for (int k = 0; k < VEC; ++k) xb[k][j] = 0.0f;
            if (s0 + j < nb) {
                load(plan[kPlanBase + s0 + j]);
#pragma unroll
                for (int k = 0; k < VEC; ++k) xb[k][j] = x[k];
            }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int k = 0; k < VEC; ++k) S[k] += xb[k][j];
    }
    float res[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        if constexpr (B1) {
            float es[THETA];
#pragma unroll
            for (int t = 0; t < THETA; ++t) es[t] = e[k][t];
            sort_registers<THETA>(es);
            float med;
            if constexpr (THETA & 1) med = es[THETA / 2];
            else med = 0.5f * (es[THETA / 2 - 1] + es[THETA / 2]);
            float best = 0.0f, bd = __builtin_huge_valf();
#pragma unroll
            for (int t = THETA - 1; t >= 0; --t) {
                S[k] += e[k][t];
                const float at = S[k] * inv_m[t];
                const float dt = fabsf(at - med);
                const bool take = dt < bd || (dt == bd && at < best);
                best = take ? at : best;
                bd = take ? dt : bd;
            }
            res[k] = best;
        } else {
            float a[THETA];
#pragma unroll
            for (int t = THETA - 1; t >= 0; --t) {
                S[k] += e[k][t];
                a[t] = S[k] * inv_m[t];
            }
            sort_registers<THETA>(e[k]);
            float med;
            if constexpr (THETA & 1) med = e[k][THETA / 2];
            else med = 0.5f * (e[k][THETA / 2 - 1] + e[k][THETA / 2]);
            res[k] = pick_closest<THETA>(a, med, beta);
        }
    }
    if (vec) {
        __builtin_nontemporal_store(floatx2{res[0], res[VEC - 1]}, reinterpret_cast<floatx2 *>(out + c));
    } else {
        out[c] = res[0];
        if (two) out[c + 1] = res[VEC - 1];
    }
}

// The general case (some round's set is not "the previous set minus its winner"); returns at once
// when the plan says the regular kernel handles the call.
template <int THETA>
__global__ __launch_bounds__(kThreads) void coord_alg1_general_kernel(
    const float *__restrict__ G, int n, int64_t d, int64_t ld, const int32_t *__restrict__ sel,
    const uint8_t *__restrict__ sets, int beta, const int32_t *__restrict__ plan, float *__restrict__ out)
{
    if (plan[kPlanRegular]) return;
    extern __shared__ float stage[];                 // [kWaves][slots][64]
    __shared__ unsigned char ops[kMaxN * kMaxN];     // slot | 0x80 if the row leaves the set
    __shared__ int off[kMaxN + 1];                   // ops of round t: [off[t], off[t+1])
    __shared__ float inv_m[kMaxN];
    __shared__ unsigned char need[kMaxN];            // row is read at all
    __shared__ unsigned char slot_of[kMaxN];         // row -> slot among the rows that are read
    __shared__ int rows[kMaxN];                      // slot -> row
    __shared__ int wslot[kMaxN];                     // slot of the winner of round t
    __shared__ int nslots;
    __shared__ int bad_flag;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    // ---- plan: which rows are read, and the signed row updates of every round -------------
    if (tid == 0) bad_flag = 0;
    if (tid < kMaxN) need[tid] = 0;
    __syncthreads();
    int my_count = 0, my_m = 0;
    if (tid < THETA) {
        for (int r = 0; r < n; ++r) {
            const int cur = sets[tid * n + r] ? 1 : 0;
            const int prev = (tid > 0 && sets[(tid - 1) * n + r]) ? 1 : 0;
            my_count += (cur != prev);
            my_m += cur;
            if (cur) need[r] = 1;
        }
        const int w = sel[tid];
        if ((unsigned)w >= (unsigned)n) bad_flag = 1;
        else need[w] = 1;
        inv_m[tid] = my_m > 0 ? 1.0f / (float)my_m : 0.0f;
        off[tid + 1] = my_count;
    }
    __syncthreads();
    if (tid == 0) {
        off[0] = 0;
        for (int t = 0; t < THETA; ++t) off[t + 1] += off[t];
        int ns = 0;
        for (int r = 0; r < n; ++r)
            if (need[r]) { slot_of[r] = (unsigned char)ns; rows[ns] = r; ++ns; }
        nslots = ns;
    }
    __syncthreads();
    if (tid < THETA) {
        int k = off[tid];
        for (int r = 0; r < n; ++r) {
            const int cur = sets[tid * n + r] ? 1 : 0;
            const int prev = (tid > 0 && sets[(tid - 1) * n + r]) ? 1 : 0;
            if (cur != prev) ops[k++] = (unsigned char)(slot_of[r] | (cur ? 0 : 0x80));
        }
        const int w = sel[tid];
        wslot[tid] = ((unsigned)w < (unsigned)n) ? slot_of[w] : 0;
    }
    __syncthreads();
    const bool bad = bad_flag != 0;
    const int U = nslots;

    const int64_t ntiles = (d + kThreads - 1) / kThreads;
    float *my = stage + (size_t)wave * U * 64;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t c = tile * kThreads + tid;
        const bool live = c < d;
        const int64_t cc = live ? c : d - 1;
        // every needed row once, all loads in flight together, then parked in LDS where the
        // update lists can index them (a lane only ever reads back what it wrote itself)
        float x[kMaxN];
#pragma unroll
        for (int s = 0; s < kMaxN; ++s)
            if (s < U) x[s] = __builtin_nontemporal_load(G + (int64_t)rows[s] * ld + cc);
#pragma unroll
        for (int s = 0; s < kMaxN; ++s)
            if (s < U) my[s * 64 + lane] = x[s];

        float e[THETA], a[THETA];
        float S = 0.0f;
#pragma unroll
        for (int t = 0; t < THETA; ++t) {
            e[t] = my[wslot[t] * 64 + lane];
            const int k1 = off[t + 1];
            for (int k = off[t]; k < k1; ++k) {
                const int op = ops[k];
                const float xv = my[(op & 63) * 64 + lane];
                S += (op & 0x80) ? -xv : xv;
            }
            a[t] = S * inv_m[t];
        }
        sort_registers<THETA>(e);
        float med;
        if constexpr (THETA & 1) med = e[THETA / 2];
        else med = 0.5f * (e[THETA / 2 - 1] + e[THETA / 2]);

        float res = pick_closest<THETA>(a, med, beta);
        if (bad) res = __int_as_float(0x7fc00000);
        if (live) out[c] = res;
    }
}

template <int THETA>
hipError_t launch_theta(const CoordAlg1Args &a, hipStream_t s)
{
    // which of the two kernels does the work is only known on the device (the plan): both are launched
    if (a.beta == 1) {
        const int64_t blocks = (a.d + 2 * kRegThreads - 1) / (2 * kRegThreads);
        coord_alg1_regular_kernel<THETA, true><<<dim3((unsigned)blocks), dim3(kRegThreads), 0, s>>>(
            a.G, a.d, a.ld, a.beta, a.plan, a.out);
    } else {
        const int64_t blocks = (a.d + kRegThreads - 1) / kRegThreads;
        coord_alg1_regular_kernel<THETA, false><<<dim3((unsigned)blocks), dim3(kRegThreads), 0, s>>>(
            a.G, a.d, a.ld, a.beta, a.plan, a.out);
    }
    const size_t lds = (size_t)kWaves * a.n * 64 * sizeof(float);   // at most n rows are parked
    const int64_t ntiles = (a.d + kThreads - 1) / kThreads;
    const int grid = (int)(ntiles < 2048 ? ntiles : 2048);
    coord_alg1_general_kernel<THETA><<<dim3(grid), dim3(kThreads), lds, s>>>(a.G, a.n, a.d, a.ld, a.sel, a.agr_sets,
                                                                            a.beta, a.plan, a.out);
    return hipGetLastError();
}

}  // namespace

#define MB_CAT2(a, b) a##b
#define MB_CAT(a, b) MB_CAT2(a, b)
#define MB_CASE(k) \
    case k: return launch_theta<8 * MB_GROUP + k>(a, s);

hipError_t MB_CAT(launch_coord_alg1_group, MB_GROUP)(const CoordAlg1Args &a, hipStream_t s)
{
    switch (a.theta - 8 * MB_GROUP) {
        MB_CASE(1) MB_CASE(2) MB_CASE(3) MB_CASE(4) MB_CASE(5) MB_CASE(6) MB_CASE(7) MB_CASE(8)
        default: return hipErrorInvalidValue;
    }
}

}  // namespace mb
