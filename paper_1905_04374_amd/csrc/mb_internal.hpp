// Internal launch interface between the C-ABI layer and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mb_coord.hpp"

namespace mb {

// ---- distance pass -------------------------------------------------------
// Layout of one block's partial results, in doubles.
//   direct: kDirectSlots = 36 row-block pairs x 64 entries
//   gram:   NT(NB) tiles x 256 entries, NB = ceil(n/16), NT = NB(NB+1)/2
constexpr int kDirectSlots = 36 * 64;
constexpr int kGramMaxBlocks = 2048;
constexpr int gram_blocks(int n) { return (n + 15) / 16; }
constexpr int gram_slots(int n) { return gram_blocks(n) * (gram_blocks(n) + 1) / 2 * 256; }
// the words the second pass of the Gram form leaves for the kernels after it, and its ticket counter
constexpr int kGateFlag = 0;    // 1: the second pass ran and its reduced tiles are to be used
constexpr int kGatePivot = 1;   // its pivot row
constexpr int kGateTicket = 2;  // workgroups of the second pass that have written their tile (zeroed by launch_reduce)

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
// max_blocks >= 1: what `partials` has room for) and reports the count.
// first_pass == null: the first pass (rows as they are).  Otherwise the second pass: first_pass =
// the reduced Gram tiles of the first; the kernel decides on the device whether it is needed,
// chooses the pivot row, leaves both in gate[kGateFlag], gate[kGatePivot] and, if needed, computes
// the Gram tiles of the rows minus the pivot row: partial tiles into `partials`, and the workgroup
// that finishes last adds them up into second_sums (so no reduction launch follows this pass).
// gate[kGateTicket] must be 0 when the second pass starts: launch_reduce of the first pass sees to it.
// prep_ordered, prep_idx (second pass only, may be null): when the pass finds that it is not needed,
// its first n workgroups leave the rows of the distance matrix ordered for the selection kernel
// (64 x 64 doubles; 2 x 64 x 64 bytes: neighbour by rank, then rank by neighbour) - see launch_select_gram.
hipError_t launch_dist_gram(const float *G, int n, int64_t d, int64_t ld, double *partials, bool bf16,
                            int max_blocks, int *nblocks, const double *first_pass, double *second_sums, int *gate,
                            double *prep_ordered, unsigned char *prep_idx, hipStream_t s);
// the same for gradients stored as 16-bit words (fmt = kStoreBf16 / kStoreFp16, ld in elements)
hipError_t launch_dist_gram_in16(const uint16_t *G, int fmt, int n, int64_t d, int64_t ld, double *partials,
                                 int max_blocks, int *nblocks, const double *first_pass, double *second_sums,
                                 int *gate, double *prep_ordered, unsigned char *prep_idx, hipStream_t s);
// partials[nblocks][stride] -> reduced[0..slots) (fixed summation order).  ticket (may be null): a
// word the kernel sets to 0 (the ticket counter of the second pass that follows).
hipError_t launch_reduce(const double *partials, int nblocks, int stride, int slots, double *reduced,
                         int *ticket, hipStream_t s);
hipError_t launch_finalize_direct(const double *reduced, int n, double *dist, int accumulate, hipStream_t s);
// Gram tiles of the first pass, of the second pass and its gate words (both null: no second pass was
// launched) -> dist[n*n]
hipError_t launch_finalize_gram(const double *reduced, const double *reduced2, const int *gate, int n, double *dist,
                                int accumulate, hipStream_t s);

// ---- selection -----------------------------------------------------------
// rounds >= 1: multi-Krum rounds; scores_out (may be null) gets the scores of the first round.
// plan (may be null; needs sel and agr_sets): kPlanWords words that get the plan of the
// Algorithm-1 coordinate pass for the result, as launch_alg1_plan(n, rounds, sel, agr_sets, plan)
// would write it.
hipError_t launch_select(const double *dist, int n, int f, int rounds, const uint8_t *active_in,
                         int32_t *sel, uint8_t *agr_sets, int32_t *m_out, double *scores_out, int32_t *plan,
                         hipStream_t s);
// The same starting from the reduced Gram tiles of the distance pass: the kernel forms the distance
// matrix itself (what launch_finalize_gram would write from the same arguments) and saves that launch.
// prep_ordered, prep_idx (may be null): what the second pass was given under these names; used when
// gate[kGateFlag] is 0 (then the second pass has filled them and the kernel skips forming and
// ordering the matrix).
hipError_t launch_select_gram(const double *reduced, const double *reduced2, const int *gate, int n, int f,
                              int rounds, int32_t *sel, uint8_t *agr_sets, int32_t *m_out, int32_t *plan,
                              const double *prep_ordered, const unsigned char *prep_idx, hipStream_t s);

// out[c] = mean over rows r with mask[r] of G[r][c]
hipError_t launch_masked_mean(const float *G, int n, int64_t d, int64_t ld, const uint8_t *mask,
                              float *out, hipStream_t s);
hipError_t launch_masked_mean_in16(const uint16_t *G, int fmt, int n, int64_t d, int64_t ld, const uint8_t *mask,
                                   float *out, hipStream_t s);

}  // namespace mb
