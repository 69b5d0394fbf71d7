// Coordinate-wise phase of multi-Bulyan exactly as Algorithm 1 prints it:
// M[c] = median over t of G^ext[t][c]; G^agr[t][c] = average of the gradients
// that round t of multi-Krum averaged; out[c] = average of the beta values
// G^agr[.][c] closest to M[c].
//
// G^agr is never materialised.  The theta x n membership matrix becomes signed
// row updates (rows entering or leaving the set from one round to the next) and
// the running sum over the current set follows them: usually a round's set is
// the previous one minus its winner, one row per round, but any membership
// matrix works.  Rows that no round uses are not read at all.  A small plan
// kernel (rowops.hip) prepares the row list and the updates; the kernel here
// reads its plan with scalar loads and keeps everything else in registers.
//
// Compiled once per group of 8 values of theta (-DMB_GROUP=0..7), and again with -DMB_IN16=1 for
// gradients stored as bf16 and -DMB_IN16=2 for fp16.
#include <hip/hip_runtime.h>

#include "mb_coord.hpp"
#include "sortnet.hpp"

#include <type_traits>

#ifndef MB_GROUP
#error "compile with -DMB_GROUP=0..7"
#endif

namespace mb {
namespace {

typedef float floatx2 __attribute__((ext_vector_type(2)));

#ifndef MB_IN16
#define MB_IN16 0   // 1 / 2: this unit holds the kernels for gradients stored as bf16 / fp16 (raw 16-bit words)
#endif
constexpr bool kIn16 = MB_IN16 != 0;
typedef typename std::conditional<kIn16, unsigned short, float>::type Elem;

// The lane's one or two coordinates of a row as they come from memory (two floats, or one word
// holding two bf16), and their fp32 values.  Kept apart so that nothing consumes a loaded value
// between two loads: the loads sit behind per-lane branches (pair or not), and a conversion right
// after one would make every load wait for the one before.
// `pair`: one load of both coordinates (8 bytes of fp32, 4 bytes of bf16; the address is aligned
// for it), `two`: there is a second coordinate at all.
template <class R>
struct RawOps;

template <>
struct RawOps<floatx2> {   // fp32 gradients
    static __device__ __forceinline__ floatx2 load(const float *p, bool pair, bool two)
    {
        if (pair) return __builtin_nontemporal_load(reinterpret_cast<const floatx2 *>(p));
        const float x0 = __builtin_nontemporal_load(p);
        return floatx2{x0, two ? __builtin_nontemporal_load(p + 1) : x0};
    }
    static __device__ __forceinline__ floatx2 zero() { return floatx2{0.0f, 0.0f}; }
    static __device__ __forceinline__ float widen(floatx2 r, int k) { return r[k]; }
    // median of coordinate k of the THETA rows, k < VEC
    template <int THETA, int VEC>
    static __device__ __forceinline__ void medians(const floatx2 (&r)[THETA], float (&med)[VEC])
    {
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            float es[THETA];
#pragma unroll
            for (int t = 0; t < THETA; ++t) es[t] = r[t][k];
            sort_registers<THETA>(es);
            if constexpr (THETA & 1) med[k] = es[THETA / 2];
            else med[k] = 0.5f * (es[THETA / 2 - 1] + es[THETA / 2]);
        }
    }
};

template <>
struct RawOps<unsigned> {   // 16-bit gradients: one word holds both
    static __device__ __forceinline__ unsigned load(const unsigned short *p, bool pair, bool two)
    {
        if (pair) return __builtin_nontemporal_load(reinterpret_cast<const unsigned *>(p));
        const unsigned lo = __builtin_nontemporal_load(p);
        const unsigned hi = two ? (unsigned)__builtin_nontemporal_load(p + 1) : lo;
        return lo | (hi << 16);
    }
    static __device__ __forceinline__ unsigned zero() { return 0u; }
    static __device__ __forceinline__ float widen(unsigned r, int k)
    {
        return widen16<(MB_IN16 == 2 ? kStoreFp16 : kStoreBf16)>(r, k != 0);
    }
    // the same, both coordinates of the words at once: sorted as two 16-bit keys per register
    // (half the comparator instructions), only the middle widened
    template <int THETA, int VEC>
    static __device__ __forceinline__ void medians(const unsigned (&r)[THETA], float (&med)[VEC])
    {
        typedef Sortable16<(MB_IN16 == 2 ? kStoreFp16 : kStoreBf16)> Key;
        typename Key::type ks[THETA];
#pragma unroll
        for (int t = 0; t < THETA; ++t) ks[t] = Key::from_word(r[t]);
        sort_registers<THETA>(ks);
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            if constexpr (THETA & 1) med[k] = widen(Key::to_word(ks[THETA / 2]), k);
            else med[k] = 0.5f * (widen(Key::to_word(ks[THETA / 2 - 1]), k) + widen(Key::to_word(ks[THETA / 2]), k));
        }
    }
};

typedef typename std::conditional<kIn16, unsigned, floatx2>::type Raw;
__device__ __forceinline__ Raw load_raw(const Elem *p, bool pair, bool two) { return RawOps<Raw>::load(p, pair, two); }
__device__ __forceinline__ Raw raw_zero() { return RawOps<Raw>::zero(); }
__device__ __forceinline__ float widen(Raw r, int k) { return RawOps<Raw>::widen(r, k); }   // coordinate k as fp32
template <int THETA, int VEC>
__device__ __forceinline__ void medians(const Raw (&r)[THETA], float (&med)[VEC])
{
    RawOps<Raw>::template medians<THETA, VEC>(r, med);
}

// One 64-bit key per average, ordered like (closeness to the median, value): the bits of the
// (non-negative) closeness above an image of the value's own bits that orders like the values
// (sign bit flipped for positive values, all bits for negative ones).
__device__ __forceinline__ unsigned long long closeness_key(float a, float med)
{
    const unsigned ua = __float_as_uint(a);
    const unsigned img = ua ^ ((unsigned)((int)ua >> 31) | 0x80000000u);
    return ((unsigned long long)__float_as_uint(fabsf(a - med)) << 32) | img;
}
__device__ __forceinline__ float key_value(unsigned long long key)
{
    const unsigned img = (unsigned)key;
    return __uint_as_float(img ^ ((img >> 31) ? 0x80000000u : 0xffffffffu));
}

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
    // ordered by (closeness, value): the first beta are the ones to average
    unsigned long long key[THETA];
#pragma unroll
    for (int p = 0; p < THETA; ++p) key[p] = closeness_key(a[p], med);
    sort_registers<THETA>(key);
    float sum = 0.0f;
#pragma unroll
    for (int p = 0; p < THETA; ++p) sum += (p < beta) ? key_value(key[p]) : 0.0f;
    return sum / (float)beta;
}

// One workgroup takes one tile and ends (measured faster than workgroups that loop over tiles,
// as in the other coordinate kernel).  The winners (slots 0 .. theta-1, kept for the median) and
// the next 16 rows are loaded in one go, further rows 16 at a time; P[t]
// accumulates the change of the running sum in round t, sum_s delta[t][s] x[s], eight slots at a
// time where the plan says something changes there.  Register arrays cannot be indexed at run
// time, so the changes are multiply-adds by -1, 0 or +1 held in scalar registers.  In the usual
// case (each round's set = the previous one minus its winner) round 0 touches every slot and every
// later round one.  The running sums S_t = P_0 + .. + P_t times 1 / |set_t| are the averages.
// SMALL = 1: beta = 1, the one average closest to the median is picked while the running sums are formed
// (SMALL = 3: beta = 2 or 3, i.e. n = 4f + 4 or 4f + 5 with the default theta: the three closest are kept)
// and a lane owns two neighbouring coordinates (8-byte loads when the rows allow it).
constexpr int kThreads = 256;
constexpr int kBatch = 16;

// the slots from B0 on, kBatch at a time (compile-time recursion over the batches)
template <int B0, int VEC, class Load, class Apply>
__device__ __forceinline__ void more_slots(int U, Load &load, Apply &apply)
{
    if constexpr (B0 < kMaxN) {
        constexpr int END = B0 + kBatch < kMaxN ? B0 + kBatch : kMaxN;
        if (B0 < U) {                                // same for every lane
            Raw yr[kBatch];
#pragma unroll
            for (int j = 0; j < END - B0; ++j) yr[j] = (B0 + j < U) ? load(B0 + j) : raw_zero();
            float y[VEC][kBatch];
#pragma unroll
            for (int j = 0; j < END - B0; ++j)
#pragma unroll
                for (int k = 0; k < VEC; ++k) y[k][j] = widen(yr[j], k);
            apply(std::integral_constant<int, B0>{}, std::integral_constant<int, END>{},
                  std::integral_constant<int, B0>{}, y);
            more_slots<END, VEC>(U, load, apply);
        }
    }
}

template <int THETA, int SMALL>
__global__ __launch_bounds__(kThreads) void coord_alg1_kernel(const Elem *__restrict__ G, int64_t d, int64_t ld,
                                                              int beta, const int32_t *__restrict__ plan,
                                                              int unless_nested, float *__restrict__ out)
{
    if (unless_nested && plan[kPlanNested]) return;   // coord_alg1_nested_kernel takes the call
    constexpr int VEC = SMALL ? 2 : 1;
    const int64_t c = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * VEC;
    if (c >= d) return;
    const bool two = VEC == 2 && c + 1 < d;
    if (plan[kPlanBad]) {
        out[c] = __int_as_float(0x7fc00000);
        if (two) out[c + 1] = __int_as_float(0x7fc00000);
        return;
    }
    const int U = plan[kPlanNSlots];
    const float *inv_m = reinterpret_cast<const float *>(plan + kPlanInvM);
    const float *delta = reinterpret_cast<const float *>(plan + kPlanDelta);
    const bool pairs_ok = VEC == 2 && ((uintptr_t)G % (2 * sizeof(Elem)) == 0) && (ld % 2 == 0) && ((uintptr_t)out % 8 == 0);
    const bool vec = pairs_ok && two;

    float e[VEC][THETA], P[VEC][THETA];
#pragma unroll
    for (int t = 0; t < THETA; ++t)
#pragma unroll
        for (int k = 0; k < VEC; ++k) P[k][t] = 0.0f;
    auto load = [&](int slot) { return load_raw(G + (int64_t)plan[kPlanRows + slot] * ld + c, vec, two); };
    // P[t] += sum over the slots [lo, hi) of delta[t][s] * v[s - base], group by group
    auto apply = [&](auto lo_c, auto hi_c, auto base_c, const auto &v) {
        constexpr int LO = decltype(lo_c)::value, HI = decltype(hi_c)::value, BASE = decltype(base_c)::value;
#pragma unroll
        for (int t = 0; t < THETA; ++t) {
            const int groups = plan[kPlanGroups + t];
#pragma unroll
            for (int g = LO / 8; g <= (HI - 1) / 8; ++g) {
                if (groups & (1 << g)) {             // same for every lane
#pragma unroll
                    for (int s2 = 8 * g; s2 < 8 * g + 8; ++s2) {
                        if (s2 >= LO && s2 < HI) {
                            const float dl = delta[t * kMaxN + s2];
#pragma unroll
                            for (int k = 0; k < VEC; ++k) P[k][t] = fmaf(dl, v[k][s2 - BASE], P[k][t]);
                        }
                    }
                }
            }
        }
    };

    // the winners (slots 0 .. theta-1, always there) and the next kBatch rows: all loads in flight at once
    constexpr int kFirstEnd = THETA + kBatch < kMaxN ? THETA + kBatch : kMaxN;
    Raw er[THETA], yr[kBatch];
#pragma unroll
    for (int t = 0; t < THETA; ++t) er[t] = load(t);
#pragma unroll
    for (int j = 0; j < kFirstEnd - THETA; ++j) yr[j] = (THETA + j < U) ? load(THETA + j) : raw_zero();
    float y[VEC][kBatch];
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
#pragma unroll
        for (int t = 0; t < THETA; ++t) e[k][t] = widen(er[t], k);
#pragma unroll
        for (int j = 0; j < kFirstEnd - THETA; ++j) y[k][j] = widen(yr[j], k);
    }
    apply(std::integral_constant<int, 0>{}, std::integral_constant<int, THETA>{}, std::integral_constant<int, 0>{}, e);
    if constexpr (kFirstEnd > THETA) {
        if (THETA < U)
            apply(std::integral_constant<int, THETA>{}, std::integral_constant<int, kFirstEnd>{},
                  std::integral_constant<int, THETA>{}, y);
    }
    // more rows than that (only with a theta below the default or a membership matrix of one's own)
    more_slots<THETA + kBatch, VEC>(U, load, apply);

    float res[VEC], meds[VEC];
    medians<THETA, VEC>(er, meds);   // of the winners' values (Algorithm 1: the median of G^ext)
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        float S = 0.0f;
        const float med = meds[k];
        if constexpr (SMALL == 1) {
            float best = 0.0f, bd = __builtin_huge_valf();
#pragma unroll
            for (int t = 0; t < THETA; ++t) {
                S += P[k][t];
                const float at = S * inv_m[t];
                const float dt = fabsf(at - med);
                const bool take = dt < bd || (dt == bd && at < best);
                best = take ? at : best;
                bd = take ? dt : bd;
            }
            res[k] = best;
        } else if constexpr (SMALL == 3) {
            // the three smallest keys so far, in order; a new one is passed down the three and what
            // falls out at the end is dropped (the same keys, hence the same choice and the same
            // order of addition, as the network of pick_closest)
            unsigned long long k0 = ~0ull, k1 = ~0ull, k2 = ~0ull;
#pragma unroll
            for (int t = 0; t < THETA; ++t) {
                S += P[k][t];
                unsigned long long x = closeness_key(S * inv_m[t], med);
                cswap(k0, x);
                cswap(k1, x);
                cswap(k2, x);
            }
            float sum = key_value(k0);
            if (THETA > 1) sum += key_value(k1);
            if (THETA > 2 && beta > 2) sum += key_value(k2);
            res[k] = sum / (float)beta;
        } else {
            float a[THETA];
#pragma unroll
            for (int t = 0; t < THETA; ++t) {
                S += P[k][t];
                a[t] = S * inv_m[t];
            }
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

// The usual case for itself, beta = 1 (the default theta with n = 4f + 3), worth a kernel of its own
// at large d: every round's set is the previous one minus its winner, so
// set_t = set_{theta-1} + {winner_t .. winner_{theta-2}} and the averages are running sums over the
// winners' values, walked from the last round back, on top of the rows of the last set (the
// slots after the winners).  No per-round accumulators: fewer registers, more waves, about 10 %
// (theta = 19) to 25 % (theta = 25) faster than the kernel above on the same input.  Does nothing
// unless the plan says the sets are nested.
constexpr int kBaseRegs = 16;   // rows of the last set loaded in one batch (the default theta leaves f <= 15)

template <int THETA>
__global__ __launch_bounds__(kThreads) void coord_alg1_nested_kernel(
    const Elem *__restrict__ G, int64_t d, int64_t ld, int beta, const int32_t *__restrict__ plan,
    float *__restrict__ out)
{
    if (!plan[kPlanNested]) return;
    constexpr int VEC = 2;
    const int64_t c = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * VEC;
    if (c >= d) return;
    const int nb = plan[kPlanNSlots] - THETA;     // rows of the last set without its winner
    const float *inv_m = reinterpret_cast<const float *>(plan + kPlanInvM);
    const bool pairs_ok = VEC == 2 && ((uintptr_t)G % (2 * sizeof(Elem)) == 0) && (ld % 2 == 0) && ((uintptr_t)out % 8 == 0);
    const bool two = VEC == 2 && c + 1 < d;
    const bool vec = pairs_ok && two;
    auto load = [&](int row) { return load_raw(G + (int64_t)row * ld + c, vec, two); };
    // all loads first (the winners' rows and one batch of the last set), conversions after
    Raw er[THETA], br[kBaseRegs];
#pragma unroll
    for (int t = 0; t < THETA; ++t) er[t] = load(plan[kPlanRows + t]);
#pragma unroll
    for (int j = 0; j < kBaseRegs; ++j) br[j] = (j < nb) ? load(plan[kPlanRows + THETA + j]) : raw_zero();
    float e[VEC][THETA];
    float S[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
#pragma unroll
        for (int t = 0; t < THETA; ++t) e[k][t] = widen(er[t], k);
        S[k] = 0.0f;
#pragma unroll
        for (int j = 0; j < kBaseRegs; ++j) S[k] += widen(br[j], k);
    }
    for (int s0 = kBaseRegs; s0 < nb; s0 += 8) {   // more rows in the last set than one batch
        Raw xr[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) xr[j] = (s0 + j < nb) ? load(plan[kPlanRows + THETA + s0 + j]) : raw_zero();
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int k = 0; k < VEC; ++k) S[k] += widen(xr[j], k);
    }
    float res[VEC], meds[VEC];
    medians<THETA, VEC>(er, meds);
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        const float med = meds[k];
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
    }
    if (vec) {
        __builtin_nontemporal_store(floatx2{res[0], res[VEC - 1]}, reinterpret_cast<floatx2 *>(out + c));
    } else {
        out[c] = res[0];
        if (two) out[c + 1] = res[VEC - 1];
    }
}

template <int THETA>
hipError_t launch_theta(const CoordAlg1Args &a, hipStream_t s)
{
    if (a.beta == 1) {
        const int64_t blocks = (a.d + 2 * kThreads - 1) / (2 * kThreads);
        // Large d: the nested-sets kernel as well; which of the two does the work is only known on
        // the device (the plan), the other returns at once.  Below, the second launch would cost
        // more than it saves.
        const int both = a.d >= (int64_t)1 << 22;
        if (both)
            coord_alg1_nested_kernel<THETA><<<dim3((unsigned)blocks), dim3(kThreads), 0, s>>>(static_cast<const Elem *>(a.G), a.d, a.ld, a.beta,
                                                                                             a.plan, a.out);
        coord_alg1_kernel<THETA, 1><<<dim3((unsigned)blocks), dim3(kThreads), 0, s>>>(static_cast<const Elem *>(a.G), a.d, a.ld, a.beta,
                                                                                       a.plan, both, a.out);
    } else if (a.beta <= 3 && THETA >= 3) {
        const int64_t blocks = (a.d + 2 * kThreads - 1) / (2 * kThreads);
        coord_alg1_kernel<THETA, 3><<<dim3((unsigned)blocks), dim3(kThreads), 0, s>>>(static_cast<const Elem *>(a.G), a.d, a.ld, a.beta,
                                                                                    a.plan, 0, a.out);
    } else {
        const int64_t blocks = (a.d + kThreads - 1) / kThreads;
        coord_alg1_kernel<THETA, 0><<<dim3((unsigned)blocks), dim3(kThreads), 0, s>>>(static_cast<const Elem *>(a.G), a.d, a.ld, a.beta,
                                                                                        a.plan, 0, a.out);
    }
    return hipGetLastError();
}

}  // namespace

#define MB_CAT2(a, b) a##b
#define MB_CAT(a, b) MB_CAT2(a, b)
#define MB_CASE(k) \
    case k: return launch_theta<8 * MB_GROUP + k>(a, s);

#if MB_IN16 == 2
hipError_t MB_CAT(launch_coord_alg1_h_group, MB_GROUP)(const CoordAlg1Args &a, hipStream_t s)
#elif MB_IN16 == 1
hipError_t MB_CAT(launch_coord_alg1_16_group, MB_GROUP)(const CoordAlg1Args &a, hipStream_t s)
#else
hipError_t MB_CAT(launch_coord_alg1_group, MB_GROUP)(const CoordAlg1Args &a, hipStream_t s)
#endif
{
    switch (a.theta - 8 * MB_GROUP) {
        MB_CASE(1) MB_CASE(2) MB_CASE(3) MB_CASE(4) MB_CASE(5) MB_CASE(6) MB_CASE(7) MB_CASE(8)
        default: return hipErrorInvalidValue;
    }
}

}  // namespace mb
