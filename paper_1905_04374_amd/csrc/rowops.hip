// Row averages: the multi-Krum output G^output = average of the m gradients of
// smallest score (Algorithm 1, function multi-Krum).  One lane owns four
// consecutive coordinates (one when the matrix is not 16-byte aligned) and
// adds the selected rows in ascending row order; the membership mask is
// uniform, so rows outside the set are skipped without being read.
// Also here: the plan of the Algorithm-1 coordinate pass (one small kernel).
#include <hip/hip_runtime.h>

#include "mb_internal.hpp"

namespace mb {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

// IN16: gradients stored as bf16 (raw 16-bit words), widened exactly in registers; VEC is then 1 or 2.
template <int VEC, bool IN16>
__global__ __launch_bounds__(256) void masked_mean_kernel(const void *__restrict__ Gv, int n, int64_t d,
                                                          int64_t ld, const uint8_t *__restrict__ mask,
                                                          float *__restrict__ out)
{
    const float *G = static_cast<const float *>(Gv);
    const unsigned short *G16 = static_cast<const unsigned short *>(Gv);
    // the membership mask as 64 bits in scalar registers (n <= 64): lane r looks at row r
    const int lane = threadIdx.x & 63;
    const unsigned long long members = __ballot(lane < n && mask[lane < n ? lane : 0] != 0);
    const int64_t c0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * VEC;
    if (c0 >= d) return;
    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.0f;
    int m = 0;
    const bool full = c0 + VEC <= d;
    // eight rows in flight at a time; the mask is the same for every lane, rows outside the set are
    // not read; members are added in ascending row order
    for (int r0 = 0; r0 < n; r0 += 8) {
        float x[8][VEC];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) x[j][e] = 0.0f;
            const int r = r0 + j;
            if (r < n && ((members >> r) & 1ull)) {
                ++m;
                if constexpr (IN16) {
                    const unsigned short *p16 = G16 + (int64_t)r * ld + c0;
                    if (VEC == 2 && full) {
                        const unsigned w = __builtin_nontemporal_load(reinterpret_cast<const unsigned *>(p16));
                        x[j][0] = __uint_as_float(w << 16);
                        x[j][1 % VEC] = __uint_as_float(w & 0xffff0000u);
                    } else {
#pragma unroll
                        for (int e = 0; e < VEC; ++e)
                            x[j][e] = (c0 + e < d) ? __uint_as_float((unsigned)p16[e] << 16) : 0.0f;
                    }
                    continue;
                }
                const float *p = G + (int64_t)r * ld + c0;
                if (VEC == 4 && full) {
                    const floatx4 v = __builtin_nontemporal_load(reinterpret_cast<const floatx4 *>(p));
                    x[j][0] = v[0]; x[j][1 % VEC] = v[1]; x[j][2 % VEC] = v[2]; x[j][3 % VEC] = v[3];
                } else {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) x[j][e] = (c0 + e < d) ? p[e] : 0.0f;
                }
            }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] += x[j][e];
    }
    const float inv = m > 0 ? 1.0f / (float)m : 0.0f;
#pragma unroll
    for (int e = 0; e < VEC; ++e)
        if (c0 + e < d) out[c0 + e] = acc[e] * inv;
}

// One wave, lane t = round t of multi-Krum (Algorithm 1).  Checks whether set_{t+1} = set_t minus
// the winner of round t for every t and writes what the two coordinate kernels need.
__global__ __launch_bounds__(64) void alg1_plan_kernel(int n, int theta, const int32_t *__restrict__ sel,
                                                       const uint8_t *__restrict__ sets,
                                                       int32_t *__restrict__ plan)
{
    __shared__ int slot_of[kMaxN];     // row -> slot, -1: no round needs the row
    __shared__ int winner[kMaxN];
    __shared__ int nslots_s;
    const int t = threadIdx.x;
    bool ok = true, bad = false;
    if (t < kMaxN) slot_of[t] = -1;
    __syncthreads();
    if (t < theta) {
        const int w = sel[t];
        const bool valid = (unsigned)w < (unsigned)n;
        bad = !valid;
        winner[t] = valid ? w : 0;
        ok = valid && sets[t * n + (valid ? w : 0)] != 0;
        int m = 0;
        for (int r = 0; r < n; ++r) {
            const int cur = sets[t * n + r] ? 1 : 0;
            m += cur;
            if (t + 1 < theta) {
                const int nxt = sets[(t + 1) * n + r] ? 1 : 0;
                ok = ok && (nxt == ((r == w) ? 0 : cur));
            }
        }
        plan[kPlanWinner + t] = valid ? w : 0;
        plan[kPlanInvM + t] = __float_as_int(m > 0 ? 1.0f / (float)m : 0.0f);
    }
    __syncthreads();
    if (t < theta) {                   // a winner that an earlier round already extracted
        for (int u = 0; u < t; ++u) bad = bad || (winner[u] == winner[t]);
    }
    const bool any_bad = __ballot(bad) != 0ull;
    const bool regular = __ballot(!ok) == 0ull && !any_bad;
    if (t == 0) {
        int nb = 0;
        const int last = winner[theta - 1];
        for (int r = 0; r < n; ++r)
            if (sets[(theta - 1) * n + r] && r != last) plan[kPlanBase + nb++] = r;
        plan[kPlanNBase] = nb;
        plan[kPlanRegular] = regular ? 1 : 0;
        plan[kPlanBad] = any_bad ? 1 : 0;
        // slots: winners first (slot t = round t), then the other rows some set contains
        int ns = 0;
        for (int u = 0; u < theta; ++u) {
            if (slot_of[winner[u]] < 0) slot_of[winner[u]] = ns;
            plan[kPlanRows + ns] = winner[u];
            ++ns;
        }
        if (!any_bad) {                // (with repeated winners the slots could run past kMaxN)
            for (int r = 0; r < n; ++r) {
                if (slot_of[r] >= 0) continue;
                bool used = false;
                for (int u = 0; u < theta; ++u) used = used || sets[u * n + r] != 0;
                if (used) {
                    slot_of[r] = ns;
                    plan[kPlanRows + ns] = r;
                    ++ns;
                }
            }
        }
        nslots_s = ns;
        plan[kPlanNSlots] = ns;
    }
    __syncthreads();
    if (t < theta) {
        const int ns = nslots_s;
        unsigned groups = 0;
        for (int s = 0; s < kMaxN; ++s) plan[kPlanDelta + t * kMaxN + s] = 0;   // 0.0f
        if (!any_bad) {
            for (int r = 0; r < n; ++r) {
                const int s = slot_of[r];
                if (s < 0 || s >= ns) continue;
                const int cur = sets[t * n + r] ? 1 : 0;
                const int prev = (t > 0 && sets[(t - 1) * n + r]) ? 1 : 0;
                if (cur != prev) {
                    plan[kPlanDelta + t * kMaxN + s] = __float_as_int(cur ? 1.0f : -1.0f);
                    groups |= 1u << (s >> 3);
                }
            }
        }
        plan[kPlanGroups + t] = (int)groups;
    }
}

}  // namespace

hipError_t launch_alg1_plan(int n, int theta, const int32_t *sel, const uint8_t *sets, int32_t *plan,
                            hipStream_t s)
{
    alg1_plan_kernel<<<dim3(1), dim3(64), 0, s>>>(n, theta, sel, sets, plan);
    return hipGetLastError();
}

hipError_t launch_masked_mean(const float *G, int n, int64_t d, int64_t ld, const uint8_t *mask,
                              float *out, hipStream_t s)
{
    const bool aligned = ((uintptr_t)G % 16 == 0) && (ld % 4 == 0);
    if (aligned)
        masked_mean_kernel<4, false><<<dim3((unsigned)((d + 1023) / 1024)), dim3(256), 0, s>>>(G, n, d, ld, mask, out);
    else
        masked_mean_kernel<1, false><<<dim3((unsigned)((d + 255) / 256)), dim3(256), 0, s>>>(G, n, d, ld, mask, out);
    return hipGetLastError();
}

hipError_t launch_masked_mean_in16(const uint16_t *G, int n, int64_t d, int64_t ld, const uint8_t *mask,
                                   float *out, hipStream_t s)
{
    const bool aligned = ((uintptr_t)G % 4 == 0) && (ld % 2 == 0);
    if (aligned)
        masked_mean_kernel<2, true><<<dim3((unsigned)((d + 511) / 512)), dim3(256), 0, s>>>(G, n, d, ld, mask, out);
    else
        masked_mean_kernel<1, true><<<dim3((unsigned)((d + 255) / 256)), dim3(256), 0, s>>>(G, n, d, ld, mask, out);
    return hipGetLastError();
}

}  // namespace mb
