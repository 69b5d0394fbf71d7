// Plan of the Algorithm-1 coordinate pass (layout in mb_internal.hpp), as a device function for
// one workgroup of NT threads: alg1_plan_kernel runs it on sets the caller supplies, select_kernel
// runs it right after its last round on the sets it has just written.
#pragma once
#include <hip/hip_runtime.h>

#include "mb_coord.hpp"

namespace mb {

// Every thread of the workgroup calls this (it goes through workgroup barriers).  A round's set
// is kept as a 64-bit mask over the rows, so nesting, sizes and the rows in use are bit operations
// of one wave (lane t = round t); the delta matrix is then filled by all threads.
template <int NT>
__device__ __forceinline__ void alg1_plan_body(int n, int theta, const int32_t *sel, const uint8_t *sets,
                                               int32_t *plan, int tid)
{
    static_assert(NT % 64 == 0 && NT >= 64 && kMaxN == 64, "lane = round = row, masks of 64 bits");
    __shared__ unsigned long long memb[kMaxN];   // bit r of memb[t]: the set of round t holds row r
    __shared__ int slot_of[kMaxN];               // row -> slot, kMaxN: no round needs the row
    __shared__ int rows[kMaxN];                  // slot -> row
    __shared__ unsigned groups[kMaxN];
    __shared__ int nslots;
    __shared__ int any_bad;
    const int lane = tid & 63, wave = tid >> 6;
    if (tid < kMaxN) { slot_of[tid] = kMaxN; groups[tid] = 0; rows[tid] = 0; }
    for (int t = wave; t < theta; t += NT / 64) {
        const unsigned long long mask = __ballot(lane < n && sets[t * n + (lane < n ? lane : 0)] != 0);
        if (lane == 0) memb[t] = mask;
    }
    __syncthreads();
    if (wave == 0) {
        const int t = lane;
        const bool live = t < theta;
        const int w0 = live ? sel[t] : 0;
        const bool valid = (unsigned)w0 < (unsigned)n;
        const int w = valid ? w0 : 0;
        const unsigned long long mine = live ? memb[t] : 0ull;
        const unsigned long long next = (t + 1 < theta) ? memb[t + 1] : 0ull;
        // nested: the winner is in its round's set, and the next set is this one without it
        bool ok = valid && ((mine >> w) & 1ull) != 0;
        if (t + 1 < theta) ok = ok && next == (mine & ~(1ull << w));
        const int m = __popcll(mine);
        if (live) {
            plan[kPlanInvM + t] = __float_as_int(m > 0 ? 1.0f / (float)m : 0.0f);
            atomicMin(&slot_of[w], t);           // winners first: slot t = round t, the first round that extracts the row
            rows[t] = w;
        }
        const bool again = live && slot_of[w] != t;   // a winner that an earlier round already extracted
        const bool bad = __ballot(live && (!valid || again)) != 0ull;
        const bool not_nested = __ballot(live && !ok) != 0ull;
        unsigned long long used = 0ull;          // rows that some round's set holds
        for (int u = 0; u < theta; ++u) used |= memb[u];
        int ns = theta;
        if (!bad) {                              // (with repeated winners the slots could run past kMaxN)
            const bool extra = lane < n && ((used >> lane) & 1ull) != 0 && slot_of[lane] == kMaxN;
            const unsigned long long ex = __ballot(extra);   // the other rows after the winners, ascending
            if (extra) {
                const int s = theta + (int)__popcll(ex & ((1ull << lane) - 1ull));
                slot_of[lane] = s;
                rows[s] = lane;
            }
            ns += (int)__popcll(ex);
        }
        if (lane == 0) {
            nslots = ns;
            any_bad = bad ? 1 : 0;
            plan[kPlanNSlots] = ns;
            plan[kPlanBad] = bad ? 1 : 0;
            plan[kPlanNested] = (!bad && !not_nested) ? 1 : 0;
        }
    }
    __syncthreads();
    const int ns = nslots;
    const bool bad = any_bad != 0;
    if (tid < kMaxN) plan[kPlanRows + tid] = tid < ns ? rows[tid] : 0;
    for (int e = tid; e < kMaxN * kMaxN; e += NT) {
        const int t = e / kMaxN, s = e % kMaxN;
        float dl = 0.0f;
        if (!bad && t < theta && s < ns) {
            const int row = rows[s];
            if (slot_of[row] == s) {             // a row counts in its first slot only
                const int cur = (int)((memb[t] >> row) & 1ull);
                const int prev = t > 0 ? (int)((memb[t - 1] >> row) & 1ull) : 0;
                dl = (float)(cur - prev);
            }
        }
        plan[kPlanDelta + e] = __float_as_int(dl);
        if (dl != 0.0f) atomicOr(&groups[t], 1u << (s >> 3));
    }
    __syncthreads();
    if (tid < kMaxN) plan[kPlanGroups + tid] = (int)groups[tid];
}

}  // namespace mb
