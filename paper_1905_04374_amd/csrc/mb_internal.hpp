// Internal launch interface between the C-ABI layer and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mb {

constexpr int kMaxN = 64;

// ---- distance pass -------------------------------------------------------
// Layout of one block's partial results, in doubles.
//   direct: kDirectSlots = 36 row-block pairs x 64 entries
//   gram:   NT(NB) tiles x 256 entries, NB = ceil(n/16), NT = NB(NB+1)/2
constexpr int kDirectSlots = 36 * 64;
constexpr int kGramMaxBlocks = 2048;
constexpr int gram_blocks(int n) { return (n + 15) / 16; }
constexpr int gram_slots(int n) { return gram_blocks(n) * (gram_blocks(n) + 1) / 2 * 256; }

// Element (i, j), i >= j, of the Gram matrix inside the reduced tile array.  Tile (I, J) holds
// rows 16I.. as the A operand and rows 16J.. as the B operand; the instruction leaves entry
// (a, b) of its 16x16 result in register a%4 of lane 16*(a/4) + b.
__device__ __forceinline__ double gram_at(const double *__restrict__ reduced, int i, int j)
{
    const int I = i >> 4, J = j >> 4, a = i & 15, b = j & 15;
    const int t = I * (I + 1) / 2 + J;
    return reduced[t * 256 + (a & 3) * 64 + 16 * (a >> 2) + b];
}

// Upper bound on the number of workgroups the distance kernels are launched with (sizes the partials).
int dist_grid_blocks(int64_t d, int algo);

hipError_t launch_dist_direct(const float *G, int n, int64_t d, int64_t ld, double *partials,
                              int nblocks, hipStream_t s);
// launches with as many workgroups as stay resident (at most dist_grid_blocks, and at most
// max_blocks >= 1: what `partials` has room for) and reports the count
hipError_t launch_dist_gram(const float *G, int n, int64_t d, int64_t ld, double *partials, bool bf16,
                            int max_blocks, int *nblocks, hipStream_t s);
// the same for gradients stored as bf16 (raw 16-bit words, ld in elements)
hipError_t launch_dist_gram_in16(const uint16_t *G, int n, int64_t d, int64_t ld, double *partials, int max_blocks,
                                 int *nblocks, hipStream_t s);
// partials[nblocks][stride] -> reduced[0..slots) (fixed summation order), then -> dist[n*n]
hipError_t launch_reduce(const double *partials, int nblocks, int stride, int slots, double *reduced,
                         hipStream_t s);
hipError_t launch_finalize_direct(const double *reduced, int n, double *dist, int accumulate, hipStream_t s);
hipError_t launch_finalize_gram(const double *reduced, int n, double *dist, int accumulate, bool canon,
                                hipStream_t s);

// ---- selection -----------------------------------------------------------
// rounds >= 1: multi-Krum rounds; scores_out (may be null) gets the scores of the first round.
// plan (may be null; needs sel and agr_sets): kPlanWords words that get the plan of the
// Algorithm-1 coordinate pass for the result, as launch_alg1_plan(n, rounds, sel, agr_sets, plan)
// would write it.
hipError_t launch_select(const double *dist, int n, int f, int rounds, const uint8_t *active_in,
                         int32_t *sel, uint8_t *agr_sets, int32_t *m_out, double *scores_out, int32_t *plan,
                         hipStream_t s);
// The same starting from the reduced Gram tiles of the distance pass: the kernel forms the distance
// matrix itself (what launch_finalize_gram would write, canon as there) and saves that launch.
hipError_t launch_select_gram(const double *reduced, bool canon, int n, int f, int rounds, int32_t *sel,
                              uint8_t *agr_sets, int32_t *m_out, int32_t *plan, hipStream_t s);

// ---- coordinate pass -----------------------------------------------------
struct CoordArgs {
    const void *G;       // fp32, or bf16 as raw 16-bit words when in16 is set
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
#define MB_DECL_GROUP(g)                                                \
    hipError_t launch_coord_group##g(const CoordArgs &a, hipStream_t s); \
    hipError_t launch_coord16_group##g(const CoordArgs &a, hipStream_t s);
MB_DECL_GROUP(0) MB_DECL_GROUP(1) MB_DECL_GROUP(2) MB_DECL_GROUP(3)
MB_DECL_GROUP(4) MB_DECL_GROUP(5) MB_DECL_GROUP(6) MB_DECL_GROUP(7)
#undef MB_DECL_GROUP

// Algorithm-1 mode: values are averages over row sets.
struct CoordAlg1Args {
    const void *G;           // fp32, or bf16 as raw 16-bit words when in16 is set
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
hipError_t launch_coord_alg1_group1(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_16_group1(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_group2(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_16_group2(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_group3(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_16_group3(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_group4(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_16_group4(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_group5(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_16_group5(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_group6(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_16_group6(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_group7(const CoordAlg1Args &a, hipStream_t s);
hipError_t launch_coord_alg1_16_group7(const CoordAlg1Args &a, hipStream_t s);

// out[c] = mean over rows r with mask[r] of G[r][c]
hipError_t launch_masked_mean(const float *G, int n, int64_t d, int64_t ld, const uint8_t *mask,
                              float *out, hipStream_t s);
hipError_t launch_masked_mean_in16(const uint16_t *G, int n, int64_t d, int64_t ld, const uint8_t *mask,
                                   float *out, hipStream_t s);

}  // namespace mb
