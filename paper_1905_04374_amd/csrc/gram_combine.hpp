// From Gram entries to squared distances (Algorithm 1, multi-Krum, the score line; Eq. 4 define the
// score on |G_i - G_j|^2 itself; the Gram form is how the distance pass evaluates it).
//
// D_ij = G_ii + G_jj - 2 G_ij carries an absolute error proportional to the norms, about
// 1e-8 (G_ii + G_jj) measured and below 1e-7 (G_ii + G_jj), whatever D_ij is.  Gradients of honest
// workers share a large common component exactly when training goes well (the hypothesis of
// Lemma 1, eta sqrt(d) sigma < |g|, says the gradient dominates its noise): norms far above the
// distances, and the form cancels.  So the first pass (rows as they are: a huge Byzantine row only
// harms its own distances) is checked pair by pair, and where some pair has
// G_ii + G_jj > kGateRatio D_ij a second pass repeats the Gram matrix on y_i = x_i - x_p, which has the
// same distances and small norms when the pivot row p lies among the bulk of the gradients.  The
// pivot is the row whose ball around it that holds half of the others is smallest (first-pass
// distances are good enough to choose it; a Byzantine row can only be chosen if it sits among the
// honest ones, where it is as good a centre as any).  Each pair then takes the value of the pass
// whose norms, i.e. whose error bound, are smaller: never worse than the first pass, and within
// 1e-7 kGateRatio D_ij = 2.6e-5 D_ij for every pair that is unflagged in either pass.
//
// Bit-identical rows have bit-identical Gram entries (G_ii = G_jj = G_ij: the same operand sequences
// enter the same instruction) and are recognised by that, not by a distance that happens to cancel:
// they are at distance exactly 0 and the later of them takes over the distance row of the first.
#pragma once
#include <hip/hip_runtime.h>

#include "mb_internal.hpp"

namespace mb {

constexpr double kGateRatio = 256.0;

struct GramTerm {
    double d;       // G_ii + G_jj - 2 G_ij, clamped at 0 (NaN stays NaN)
    double norms;   // G_ii + G_jj: the error of d is proportional to it
    bool same;      // the three entries are bit-identical: the rows are copies of each other
};

__device__ __forceinline__ GramTerm gram_term(const double *__restrict__ R, int hi, int lo)
{
    const double a = gram_at(R, hi, hi), b = gram_at(R, lo, lo), c = gram_at(R, hi, lo);
    GramTerm t;
    t.same = (a == b) && (a == c);
    t.norms = a + b;
    const double v = t.norms - 2.0 * c;
    t.d = v < 0.0 ? 0.0 : v;
    return t;
}

// a pair the first pass cannot be trusted on
__device__ __forceinline__ bool gram_flagged(const GramTerm &t)
{
    return !t.same && t.norms > kGateRatio * t.d;   // false whenever something is NaN
}

// squared distance of rows hi > lo from the first pass (R1) and, if it ran, the second (R2)
__device__ __forceinline__ double gram_pair_distance(const double *__restrict__ R1,
                                                     const double *__restrict__ R2, bool refined, int hi,
                                                     int lo)
{
    const GramTerm t1 = gram_term(R1, hi, lo);
    if (t1.same || !refined) return t1.d;
    const GramTerm t2 = gram_term(R2, hi, lo);
    return t2.norms < t1.norms ? t2.d : t1.d;
}

}  // namespace mb
