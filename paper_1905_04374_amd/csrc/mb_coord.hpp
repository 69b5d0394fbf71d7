// Internal launch interface of the coordinate-pass kernels (the files that are compiled once per
// group of theta values include only this header, so that changes elsewhere do not rebuild them).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mb {

constexpr int kMaxN = 64;

// How the gradients are stored: fp32, or 16-bit words (bf16 = the upper half of the fp32 pattern; IEEE
// fp16).  Both 16-bit formats widen exactly to fp32 in registers; everything computed from them is
// fp32 / fp64 as for fp32 gradients.
enum Storage { kStoreFp32 = 0, kStoreBf16 = 1, kStoreFp16 = 2 };

// the 16-bit value in the low (hi = false) or high half of w, as fp32
template <int FMT>
__device__ __forceinline__ float widen16(unsigned w, bool hi)
{
    static_assert(FMT == kStoreBf16 || FMT == kStoreFp16, "a 16-bit format");
    if constexpr (FMT == kStoreBf16) {
        return __uint_as_float(hi ? (w & 0xffff0000u) : (w << 16));
    } else {
        const unsigned short h = (unsigned short)(hi ? (w >> 16) : (w & 0xffffu));
        return (float)__builtin_bit_cast(_Float16, h);
    }
}

// A word of two 16-bit values as two keys that sort like the values, and back.  fp16: the values
// themselves (packed half min / max).  bf16 has no packed min / max: sign-magnitude bits become
// two's-complement integers of the same order (negative values get their magnitude bits inverted);
// the map is its own inverse.  (-0 sorts before +0: equal values either way.)
template <int FMT>
struct Sortable16;
template <>
struct Sortable16<kStoreFp16> {
    typedef _Float16 type __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ type from_word(unsigned w) { return __builtin_bit_cast(type, w); }
    static __device__ __forceinline__ unsigned to_word(type k) { return __builtin_bit_cast(unsigned, k); }
};
template <>
struct Sortable16<kStoreBf16> {
    typedef short type __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ type flip(type x)
    {
        const type mask = {0x7fff, 0x7fff};
        return x ^ ((x >> 15) & mask);
    }
    static __device__ __forceinline__ type from_word(unsigned w) { return flip(__builtin_bit_cast(type, w)); }
    static __device__ __forceinline__ unsigned to_word(type k) { return __builtin_bit_cast(unsigned, flip(k)); }
};

// ---- coordinate pass -----------------------------------------------------
struct CoordArgs {
    const void *G;       // fp32, or raw 16-bit words when in16 is kStoreBf16 / kStoreFp16
    int n;
    int64_t d;
    int64_t ld;
    const int32_t *sel;  // theta row indices, or null = rows 0..theta-1
    int theta;
    int beta;            // number of averaged values; ignored when median_only
    int median_only;     // output the median itself
    float *out;
    int in16;
};
hipError_t launch_coord_selected(const CoordArgs &a, hipStream_t s);
// one per translation unit, covering theta in [8g+1, 8g+8]
#define MB_DECL_GROUP(g)                                                  \
    hipError_t launch_coord_group##g(const CoordArgs &a, hipStream_t s);   \
    hipError_t launch_coord16_group##g(const CoordArgs &a, hipStream_t s); \
    hipError_t launch_coordh_group##g(const CoordArgs &a, hipStream_t s);
MB_DECL_GROUP(0) MB_DECL_GROUP(1) MB_DECL_GROUP(2) MB_DECL_GROUP(3)
MB_DECL_GROUP(4) MB_DECL_GROUP(5) MB_DECL_GROUP(6) MB_DECL_GROUP(7)
#undef MB_DECL_GROUP

// Algorithm-1 mode: values are averages over row sets.
struct CoordAlg1Args {
    const void *G;           // fp32, or raw 16-bit words when in16 is kStoreBf16 / kStoreFp16
    int n;
    int64_t d;
    int64_t ld;
    const int32_t *sel;      // theta winners
    const uint8_t *agr_sets; // theta x n
    int theta;
    int beta;
    float *out;
    int32_t *plan;           // kPlanWords words, written by launch_alg1_plan or by the selection
    int in16;
};
// Plan of the Algorithm-1 coordinate pass (int32 words), written by launch_alg1_plan or, for its
// own result, by launch_select.
// Every row that some round needs gets a slot: the winner of round t in slot t, the other rows
// after them in ascending order (nslots in all).  delta[t][s] in {-1, 0, +1} (float bits) is the
// change of slot s's membership from round t-1 to round t (round -1: the empty set), groups[t] has
// bit g set when delta[t][8g .. 8g+7] is not all zero, inv_m[t] = 1 / |set_t| (float bits).
// bad: an index out of range or repeated.  nested: every round's set is the previous one minus
// its winner (then the slots after the winners are the last set without its winner).
constexpr int kPlanNSlots = 0;
constexpr int kPlanBad = 1;
constexpr int kPlanNested = 2;
constexpr int kPlanInvM = 3;
constexpr int kPlanRows = kPlanInvM + kMaxN;
constexpr int kPlanGroups = kPlanRows + kMaxN;
constexpr int kPlanDelta = kPlanGroups + kMaxN;
constexpr int kPlanWords = kPlanDelta + kMaxN * kMaxN;
hipError_t launch_alg1_plan(int n, int theta, const int32_t *sel, const uint8_t *sets, int32_t *plan,
                            hipStream_t s);
hipError_t launch_coord_alg1(const CoordAlg1Args &a, hipStream_t s);
// one per translation unit, covering theta in [8g+1, 8g+8]
hipError_t launch_coord_alg1_group0(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_16_group0(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_h_group0(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_group1(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_16_group1(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_h_group1(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_group2(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_16_group2(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_h_group2(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_group3(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_16_group3(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_h_group3(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_group4(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_16_group4(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_h_group4(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_group5(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_16_group5(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_h_group5(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_group6(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_16_group6(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_h_group6(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_group7(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_16_group7(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_h_group7(const CoordAlg1Args &a, hipStream_t s);

}  // namespace mb
