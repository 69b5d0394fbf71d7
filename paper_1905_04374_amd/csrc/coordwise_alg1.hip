// Coordinate-wise phase of multi-Bulyan exactly as Algorithm 1 prints it:
// M[c] = median over t of G^ext[t][c]; G^agr[t][c] = average of the gradients
// that round t of multi-Krum averaged; out[c] = average of the beta values
// G^agr[.][c] closest to M[c].
//
// G^agr is never materialised.  Consecutive rounds average almost the same
// set of gradients, so each workgroup first turns the theta x n membership
// matrix into a list of signed row updates (rows entering or leaving the set
// from one round to the next); the running sum S_t = S_{t-1} +- few rows then
// costs a handful of adds per round.  A wave stages the values of the rows it
// needs for its 64 coordinates in LDS (row-major, lane = coordinate), because
// the update lists index rows at run time.  Rows that no round uses are not
// read at all.
//
// Compiled once per group of 16 values of theta (-DMB_GROUP=0..3).
#include <hip/hip_runtime.h>

#include "mb_internal.hpp"
#include "sortnet.hpp"

#ifndef MB_GROUP
#error "compile with -DMB_GROUP=0..3"
#endif

namespace mb {
namespace {

constexpr int kThreads = 128;   // 2 waves: the staging area is n x 256 bytes per wave
constexpr int kWaves = kThreads / 64;

template <int THETA>
__global__ __launch_bounds__(kThreads) void coord_alg1_kernel(
    const float *__restrict__ G, int n, int64_t d, int64_t ld, const int32_t *__restrict__ sel,
    const uint8_t *__restrict__ sets, int beta, float *__restrict__ out)
{
    extern __shared__ float stage[];                 // [kWaves][n][64]
    __shared__ unsigned char ops[kMaxN * kMaxN];     // row | 0x80 if the row leaves the set
    __shared__ int off[kMaxN + 1];                   // ops of round t: [off[t], off[t+1])
    __shared__ float inv_m[kMaxN];
    __shared__ unsigned char need[kMaxN];            // row is read at all
    __shared__ int winner[kMaxN];
    __shared__ int bad_flag;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    // ---- plan: signed row updates per round --------------------------------
    if (tid == 0) bad_flag = 0;
    if (tid < n) need[tid] = 0;
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
        if ((unsigned)w >= (unsigned)n) { bad_flag = 1; winner[tid] = 0; }
        else { winner[tid] = w; need[w] = 1; }
        inv_m[tid] = my_m > 0 ? 1.0f / (float)my_m : 0.0f;
        off[tid + 1] = my_count;
    }
    __syncthreads();
    if (tid == 0) {
        off[0] = 0;
        for (int t = 0; t < THETA; ++t) off[t + 1] += off[t];
    }
    __syncthreads();
    if (tid < THETA) {
        int k = off[tid];
        for (int r = 0; r < n; ++r) {
            const int cur = sets[tid * n + r] ? 1 : 0;
            const int prev = (tid > 0 && sets[(tid - 1) * n + r]) ? 1 : 0;
            if (cur != prev) ops[k++] = (unsigned char)(r | (cur ? 0 : 0x80));
        }
    }
    __syncthreads();
    const bool bad = bad_flag != 0;

    float *my = stage + (size_t)wave * n * 64;
    const int64_t ntiles = (d + kThreads - 1) / kThreads;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t c = tile * kThreads + tid;
        const bool live = c < d;
        // stage the needed rows of this wave's 64 coordinates
        for (int r = 0; r < n; ++r)
            if (need[r]) my[r * 64 + lane] = live ? G[(int64_t)r * ld + c] : 0.0f;
        // (a wave only reads what it wrote itself: no workgroup barrier needed, LDS
        //  operations of one wave complete in order)
        float e[THETA], a[THETA];
        float S = 0.0f;
#pragma unroll
        for (int t = 0; t < THETA; ++t) {
            e[t] = my[winner[t] * 64 + lane];
            const int k1 = off[t + 1];
            for (int k = off[t]; k < k1; ++k) {
                const int op = ops[k];
                const float x = my[(op & 63) * 64 + lane];
                S += (op & 0x80) ? -x : x;
            }
            a[t] = S * inv_m[t];
        }
        sort_registers<THETA>(e);
        float med;
        if constexpr (THETA & 1) med = e[THETA / 2];
        else med = 0.5f * (e[THETA / 2 - 1] + e[THETA / 2]);

        float res;
        if (beta == 1) {
            // the value closest to the median; equal closeness: the smaller value
            float best = a[0], bd = fabsf(a[0] - med);
#pragma unroll
            for (int t = 1; t < THETA; ++t) {
                const float dt = fabsf(a[t] - med);
                const bool take = dt < bd || (dt == bd && a[t] < best);
                best = take ? a[t] : best;
                bd = take ? dt : bd;
            }
            res = best;
        } else {
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
            res = sum / (float)beta;
        }
        if (bad) res = __int_as_float(0x7fc00000);
        if (live) out[c] = res;
    }
}

template <int THETA>
hipError_t launch_theta(const CoordAlg1Args &a, hipStream_t s)
{
    const size_t lds = (size_t)kWaves * a.n * 64 * sizeof(float);
    const int64_t ntiles = (a.d + kThreads - 1) / kThreads;
    const int grid = (int)(ntiles < 2048 ? ntiles : 2048);
    coord_alg1_kernel<THETA><<<dim3(grid), dim3(kThreads), lds, s>>>(a.G, a.n, a.d, a.ld, a.sel, a.agr_sets,
                                                                     a.beta, a.out);
    return hipGetLastError();
}

}  // namespace

#define MB_CAT2(a, b) a##b
#define MB_CAT(a, b) MB_CAT2(a, b)
#define MB_CASE(k) \
    case k: return launch_theta<16 * MB_GROUP + k>(a, s);

hipError_t MB_CAT(launch_coord_alg1_group, MB_GROUP)(const CoordAlg1Args &a, hipStream_t s)
{
    switch (a.theta - 16 * MB_GROUP) {
        MB_CASE(1) MB_CASE(2) MB_CASE(3) MB_CASE(4) MB_CASE(5) MB_CASE(6) MB_CASE(7) MB_CASE(8)
        MB_CASE(9) MB_CASE(10) MB_CASE(11) MB_CASE(12) MB_CASE(13) MB_CASE(14) MB_CASE(15) MB_CASE(16)
        default: return hipErrorInvalidValue;
    }
}

}  // namespace mb
