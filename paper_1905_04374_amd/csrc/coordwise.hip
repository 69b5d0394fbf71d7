// Coordinate-wise phase of multi-Bulyan (Algorithm 1, multi-Bulyan, after the
// loop; Section II-B): per coordinate, the median of the theta extracted
// values, the beta values closest to it, their average.
//
// One lane owns VEC consecutive coordinates.  It loads the theta values of
// each (theta coalesced row streams per wave, 8-byte non-temporal loads when aligned),
// sorts them in registers with a compile-time network and picks the window
// around the median.  Nothing is staged in LDS: the working set is theta
// floats per coordinate and fits the register file for theta <= 64.
//
// This file is compiled once per group of 8 values of theta (-DMB_GROUP=g), and again with
// -DMB_IN16=1 for gradients stored as bf16 and -DMB_IN16=2 for fp16; there a lane's two
// coordinates arrive in one word and are sorted side by side as two 16-bit keys per register.
#include <hip/hip_runtime.h>

#include "mb_coord.hpp"
#include "sortnet.hpp"

#ifndef MB_GROUP
#error "compile with -DMB_GROUP=0..7"
#endif

namespace mb {
namespace {

constexpr float kInf = __builtin_huge_valf();

// v ascending.  K = number of values to take besides the median itself (odd THETA: beta-1; even:
// beta).  Candidates: left L[a] = v[H-1-a], right R[b] = v[H+ODD+b]; order by (distance to the
// median, left before right).  WIN = candidates per side the caller may need (K <= WIN).
template <int THETA, int WIN>
__device__ __forceinline__ float closest_sum(const float (&v)[THETA], int K, bool median_only)
{
    constexpr bool ODD = (THETA & 1) != 0;
    constexpr int H = THETA / 2;
    float med;
    if constexpr (ODD) med = v[H];
    else med = 0.5f * (v[H - 1] + v[H]);
    if (median_only) return med;
    float sum = ODD ? med : 0.0f;
    if constexpr (H > 0) {
        if constexpr (WIN < H || H <= 3) {
            // greedy two-sided walk held in shift registers (small windows)
            constexpr int W = WIN < H ? WIN : H;
            constexpr int STEPS = WIN < H ? WIN : 2 * H;   // a limited window is only used with K <= WIN
            float L[W + 1], R[W + 1];
#pragma unroll
            for (int a = 0; a < W; ++a) {
                L[a] = v[H - 1 - a];
                R[a] = v[H + (ODD ? 1 : 0) + a];
            }
            L[W] = -kInf;
            R[W] = kInf;
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                if (s < K) {
                    const float dl = med - L[0];
                    const float dr = R[0] - med;
                    const bool left = dl <= dr;      // equal closeness: the smaller value
                    sum += left ? L[0] : R[0];
#pragma unroll
                    for (int a = 0; a < W; ++a) {
                        L[a] = left ? L[a + 1] : L[a];
                        R[a] = left ? R[a] : R[a + 1];
                    }
                }
            }
        } else {
            // How many of the K closest lie on the left.  Both sides are ordered by their distance to
            // the median, so left candidate a is among the K closest iff fewer than K - a right ones
            // are strictly closer, i.e. iff a < K and not dR[K-1-a] < dL[a] (a right candidate past
            // the end counts as infinitely far).  K is the same for every lane: E[a] = dR[K-1-a] is
            // the right-hand distances reversed and shifted by a uniform amount, done by a barrel
            // shifter of log2(2H) stages of selects on a scalar condition - O(H log H) where
            // counting over all pairs takes H^2.
            constexpr int N2 = 2 * H;
            constexpr int STAGES = N2 <= 2 ? 1 : N2 <= 4 ? 2 : N2 <= 8 ? 3 : N2 <= 16 ? 4 : N2 <= 32 ? 5 : N2 <= 64 ? 6 : 7;
            float dL[H], Y[N2 + (1 << STAGES)];
#pragma unroll
            for (int a = 0; a < H; ++a) dL[a] = med - v[H - 1 - a];
            // Y[j] = X[2H-1-j], X[m] = dR[m] for m < H and +inf beyond; E[a] = X[K-1-a] = Y[a + (2H - K)]
#pragma unroll
            for (int j = 0; j < N2 + (1 << STAGES); ++j) {
                const int m = N2 - 1 - j;
                Y[j] = (m >= 0 && m < H) ? v[H + (ODD ? 1 : 0) + m] - med : kInf;
            }
            const int shift = N2 - K;            // 0 .. 2H, uniform
#pragma unroll
            for (int st = 0; st < STAGES; ++st) {
                const bool on = ((shift >> st) & 1) != 0;
#pragma unroll
                for (int j = 0; j < N2; ++j) Y[j] = on ? Y[j + (1 << st)] : Y[j];
            }
            int na = 0;
#pragma unroll
            for (int a = 0; a < H; ++a) na += (a < K && !(Y[a] < dL[a])) ? 1 : 0;
            const int nb = K - na;
#pragma unroll
            for (int a = 0; a < H; ++a) sum += (a < na) ? v[H - 1 - a] : 0.0f;
#pragma unroll
            for (int b = 0; b < H; ++b) sum += (b < nb) ? v[H + (ODD ? 1 : 0) + b] : 0.0f;
        }
    }
    return sum;
}

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

#ifndef MB_IN16
#define MB_IN16 0   // 1 / 2: this unit holds the kernels for gradients stored as bf16 / fp16
#endif

// FMT != kStoreFp32: the gradients are raw 16-bit words (bf16 or fp16); they widen exactly to fp32 in
// registers and the arithmetic and the output stay fp32.
template <int THETA, int VEC, int WIN, int FMT>
__global__ __launch_bounds__(256) void coord_selected_kernel(
    const void *__restrict__ Gv, int n, int64_t d, int64_t ld, const int32_t *__restrict__ sel,
    int K, int median_only, float scale, float *__restrict__ out)
{
    const float *G = static_cast<const float *>(Gv);
    const unsigned short *G16 = static_cast<const unsigned short *>(Gv);
    const int64_t c0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * VEC;
    if (c0 >= d) return;
    // row offsets of the theta extracted gradients (uniform: scalar loads), validated
    int64_t roff[THETA];
    bool bad = false;
#pragma unroll
    for (int t = 0; t < THETA; ++t) {
        int r = sel ? sel[t] : t;
        if ((unsigned)r >= (unsigned)n) { bad = true; r = 0; }
        roff[t] = (int64_t)r * ld;
    }
    float v[VEC][THETA];
    const bool full = (c0 + VEC <= d);
    if constexpr (FMT != kStoreFp32) {
        static_assert(VEC <= 2, "16-bit input: one or two coordinates per lane");
        if (VEC == 2 && full) {
            // one word holds the lane's two coordinates: they are sorted side by side, as two 16-bit
            // keys per register (half the comparator instructions), and only what the window around
            // the median needs is widened afterwards
            typedef Sortable16<FMT> Key;
            typename Key::type k[THETA];
#pragma unroll
            for (int t = 0; t < THETA; ++t)
                k[t] = Key::from_word(__builtin_nontemporal_load(reinterpret_cast<const unsigned *>(G16 + roff[t] + c0)));
            sort_registers<THETA>(k);
            float res2[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                float w[THETA];
#pragma unroll
                for (int t = 0; t < THETA; ++t) w[t] = widen16<FMT>(Key::to_word(k[t]), e == 1);
                res2[e] = closest_sum<THETA, WIN>(w, K, median_only != 0) * scale;
                if (bad) res2[e] = __int_as_float(0x7fc00000);
            }
            const floatx2 o = {res2[0], res2[1]};
            __builtin_nontemporal_store(o, reinterpret_cast<floatx2 *>(out + c0));
            return;
        } else {
#pragma unroll
            for (int t = 0; t < THETA; ++t)
#pragma unroll
                for (int e = 0; e < VEC; ++e)
                    v[e][t] = (c0 + e < d) ? widen16<FMT>((unsigned)G16[roff[t] + c0 + e], false) : 0.0f;
        }
    } else if (VEC == 4 && full) {
        // the input is read once and never again: non-temporal loads keep it from displacing
        // anything useful in the caches
#pragma unroll
        for (int t = 0; t < THETA; ++t) {
            const floatx4 x = __builtin_nontemporal_load(reinterpret_cast<const floatx4 *>(G + roff[t] + c0));
            v[0][t] = x.x; v[1 % VEC][t] = x.y; v[2 % VEC][t] = x.z; v[3 % VEC][t] = x.w;
        }
    } else if (VEC == 2 && full) {
#pragma unroll
        for (int t = 0; t < THETA; ++t) {
            const floatx2 x = __builtin_nontemporal_load(reinterpret_cast<const floatx2 *>(G + roff[t] + c0));
            v[0][t] = x.x; v[1 % VEC][t] = x.y;
        }
    } else if (VEC == 1) {
#pragma unroll
        for (int t = 0; t < THETA; ++t) v[0][t] = __builtin_nontemporal_load(G + roff[t] + c0);
    } else {
#pragma unroll
        for (int t = 0; t < THETA; ++t)
#pragma unroll
            for (int e = 0; e < VEC; ++e) v[e][t] = (c0 + e < d) ? G[roff[t] + c0 + e] : 0.0f;
    }
    float res[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        sort_registers<THETA>(v[e]);
        res[e] = closest_sum<THETA, WIN>(v[e], K, median_only != 0) * scale;
        if (bad) res[e] = __int_as_float(0x7fc00000);
    }
    if (VEC == 4 && full) {
        const floatx4 o = {res[0], res[1 % VEC], res[2 % VEC], res[3 % VEC]};
        __builtin_nontemporal_store(o, reinterpret_cast<floatx4 *>(out + c0));
        return;
    }
    if (VEC == 2 && full) {
        const floatx2 o = {res[0], res[1 % VEC]};
        __builtin_nontemporal_store(o, reinterpret_cast<floatx2 *>(out + c0));
        return;
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e)
        if (c0 + e < d) out[c0 + e] = res[e];
}

template <int THETA>
hipError_t launch_theta(const CoordArgs &a, hipStream_t s)
{
    constexpr bool ODD = (THETA & 1) != 0;
    constexpr int H = THETA / 2;
    const int K = a.median_only ? 0 : a.beta - (ODD ? 1 : 0);
    const float scale = a.median_only ? 1.0f : 1.0f / (float)a.beta;
    // two coordinates per lane (8-byte loads; 4-byte loads of bf16 pairs) measured faster than four
    // at every theta tried (11, 15, 21, 27): fewer live registers, more waves in flight
    constexpr int FMT = MB_IN16;
    const bool aligned = ((uintptr_t)a.G % (FMT != kStoreFp32 ? 4 : 8) == 0) && ((uintptr_t)a.out % 8 == 0) && (a.ld % 2 == 0);
    const dim3 block(256);
    if (aligned) {
        const dim3 grid((unsigned)((a.d + 511) / 512));
        if (K <= 2 && H > 2)
            coord_selected_kernel<THETA, 2, 2, FMT><<<grid, block, 0, s>>>(a.G, a.n, a.d, a.ld, a.sel, K,
                                                                            a.median_only, scale, a.out);
        else if (K <= 4 && H > 4)   // beta = 4 or 5 (n = 4f + 4, 4f + 5): still a window of the network's middle
            coord_selected_kernel<THETA, 2, 4, FMT><<<grid, block, 0, s>>>(a.G, a.n, a.d, a.ld, a.sel, K,
                                                                            a.median_only, scale, a.out);
        else
            coord_selected_kernel<THETA, 2, (H > 0 ? H : 1), FMT><<<grid, block, 0, s>>>(
                a.G, a.n, a.d, a.ld, a.sel, K, a.median_only, scale, a.out);
    } else {
        // one coordinate per lane, element loads; the same windows as above, so that a result does
        // not depend on how the matrix happens to be aligned (the windows add in different orders)
        const dim3 grid((unsigned)((a.d + 255) / 256));
        if (K <= 2 && H > 2)
            coord_selected_kernel<THETA, 1, 2, FMT><<<grid, block, 0, s>>>(a.G, a.n, a.d, a.ld, a.sel, K,
                                                                            a.median_only, scale, a.out);
        else if (K <= 4 && H > 4)
            coord_selected_kernel<THETA, 1, 4, FMT><<<grid, block, 0, s>>>(a.G, a.n, a.d, a.ld, a.sel, K,
                                                                            a.median_only, scale, a.out);
        else
            coord_selected_kernel<THETA, 1, (H > 0 ? H : 1), FMT><<<grid, block, 0, s>>>(
                a.G, a.n, a.d, a.ld, a.sel, K, a.median_only, scale, a.out);
    }
    return hipGetLastError();
}

}  // namespace

#define MB_CAT2(a, b) a##b
#define MB_CAT(a, b) MB_CAT2(a, b)

#if MB_IN16 == 2
hipError_t MB_CAT(launch_coordh_group, MB_GROUP)(const CoordArgs &a, hipStream_t s)
#elif MB_IN16 == 1
hipError_t MB_CAT(launch_coord16_group, MB_GROUP)(const CoordArgs &a, hipStream_t s)
#else
hipError_t MB_CAT(launch_coord_group, MB_GROUP)(const CoordArgs &a, hipStream_t s)
#endif
{
    switch (a.theta - 8 * MB_GROUP) {
        case 1: return launch_theta<8 * MB_GROUP + 1>(a, s);
        case 2: return launch_theta<8 * MB_GROUP + 2>(a, s);
        case 3: return launch_theta<8 * MB_GROUP + 3>(a, s);
        case 4: return launch_theta<8 * MB_GROUP + 4>(a, s);
        case 5: return launch_theta<8 * MB_GROUP + 5>(a, s);
        case 6: return launch_theta<8 * MB_GROUP + 6>(a, s);
        case 7: return launch_theta<8 * MB_GROUP + 7>(a, s);
        case 8: return launch_theta<8 * MB_GROUP + 8>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace mb
