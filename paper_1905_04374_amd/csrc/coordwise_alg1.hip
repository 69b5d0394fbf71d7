// Coordinate-wise phase of multi-Bulyan exactly as Algorithm 1 prints it:
// M[c] = median over t of G^ext[t][c]; G^agr[t][c] = average of the gradients
// that round t of multi-Krum averaged; out[c] = average of the beta values
// G^agr[.][c] closest to M[c].
//
// G^agr is never materialised.  In the regular case a round's set is the
// previous one minus its winner; the averages are then running sums over the
// winners' values (needed for the median anyway) on top of the last round's
// set: theta + f row streams, all in registers.  Otherwise (the order of the
// scores changed between rounds) the theta x n membership matrix becomes signed
// row updates (rows entering or leaving the set from one round to the next) and
// the running sum S_t = S_{t-1} +- few rows follows them; rows that no round
// uses are not read at all.  A small plan kernel (rowops.hip) decides which case
// holds and prepares both; the two kernels here read its plan with scalar loads.
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
// when the plan says the regular kernel handles the call.  Every row that some round needs has a
// slot (the winner of round t in slot t), a lane holds its coordinate of all of them in registers,
// and the running sum over the current set follows the plan's signed membership changes:
// S_t = S_{t-1} + sum_s delta[t][s] x[s].  Register arrays cannot be indexed at run time, so the
// changes are applied as multiply-adds by -1, 0 or +1 from scalar registers, in groups of eight
// slots that are skipped when nothing in them changes (after round 0 only a few rows move).
template <int THETA>
__global__ __launch_bounds__(kRegThreads) void coord_alg1_general_kernel(
    const float *__restrict__ G, int64_t d, int64_t ld, int beta, const int32_t *__restrict__ plan,
    float *__restrict__ out)
{
    if (plan[kPlanRegular]) return;
    const int64_t c = (int64_t)blockIdx.x * kRegThreads + threadIdx.x;
    if (c >= d) return;
    if (plan[kPlanBad]) {
        out[c] = __int_as_float(0x7fc00000);
        return;
    }
    const int U = plan[kPlanNSlots];
    const float *inv_m = reinterpret_cast<const float *>(plan + kPlanInvM);
    const float *delta = reinterpret_cast<const float *>(plan + kPlanDelta);
    float x[kMaxN];
#pragma unroll
    for (int s = 0; s < kMaxN; ++s) {
        x[s] = 0.0f;
        if (s < U) x[s] = __builtin_nontemporal_load(G + (int64_t)plan[kPlanRows + s] * ld + c);
    }
    float e[THETA], a[THETA];
    float S = 0.0f;
#pragma unroll
    for (int t = 0; t < THETA; ++t) {
        e[t] = x[t];
        const int groups = plan[kPlanGroups + t];
#pragma unroll
        for (int g = 0; g < kMaxN / 8; ++g) {
            if (groups & (1 << g)) {           // same for every lane
#pragma unroll
                for (int j = 0; j < 8; ++j) S = fmaf(delta[t * kMaxN + 8 * g + j], x[8 * g + j], S);
            }
        }
        a[t] = S * inv_m[t];
    }
    sort_registers<THETA>(e);
    float med;
    if constexpr (THETA & 1) med = e[THETA / 2];
    else med = 0.5f * (e[THETA / 2 - 1] + e[THETA / 2]);
    out[c] = pick_closest<THETA>(a, med, beta);
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
    const int64_t gblocks = (a.d + kRegThreads - 1) / kRegThreads;
    coord_alg1_general_kernel<THETA><<<dim3((unsigned)gblocks), dim3(kRegThreads), 0, s>>>(a.G, a.d, a.ld, a.beta,
                                                                                          a.plan, a.out);
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
