// Row averages: the multi-Krum output G^output = average of the m gradients of
// smallest score (Algorithm 1, function multi-Krum).  One lane owns four
// consecutive coordinates (one when the matrix is not 16-byte aligned) and
// adds the selected rows in ascending row order; the membership mask is
// uniform, so rows outside the set are skipped without being read.
// Also here: the plan of the Algorithm-1 coordinate pass (one small kernel).
#include <hip/hip_runtime.h>

#include "alg1_plan.hpp"
#include "mb_internal.hpp"

namespace mb {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

// Row loads in flight per lane (kRows) and coordinates per lane, fp32: 8 rows of 16 bytes each up to 2^24
// coordinates, 32 rows of 8 bytes beyond (measured at n = 39: 0.194 against 0.200 ms at d = 1e7, 5.1 against
// 4.9 ms at d = 2.5e8).  16-bit storage: 8 rows of one word.
constexpr int kRowsDefault = 8, kRowsLarge = 32;

// FMT != kStoreFp32: gradients stored as raw 16-bit words (bf16 or fp16), widened exactly in registers;
// VEC is then 1 or 2.
template <int VEC, int FMT, int kRows>
__global__ __launch_bounds__(256) void masked_mean_kernel(const void *__restrict__ Gv, int n, int64_t d,
                                                          int64_t ld, const uint8_t *__restrict__ mask,
                                                          float *__restrict__ out)
{
    constexpr bool IN16 = FMT != kStoreFp32;
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
    // kRows rows in flight at a time; the mask is the same for every lane, rows outside the set are
    // not read; members are added in ascending row order
    for (int r0 = 0; r0 < n; r0 += kRows) {
        float x[kRows][VEC];
        unsigned raw[kRows];   // bf16: the words as loaded; widened after the batch is out, so that no
                           // load waits for the conversion of the one before
#pragma unroll
        for (int j = 0; j < kRows; ++j) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) x[j][e] = 0.0f;
            raw[j] = 0u;
            const int r = r0 + j;
            if (r < n && ((members >> r) & 1ull)) {
                ++m;
                if constexpr (IN16) {
                    const unsigned short *p16 = G16 + (int64_t)r * ld + c0;
                    if (VEC == 2 && full) {
                        raw[j] = __builtin_nontemporal_load(reinterpret_cast<const unsigned *>(p16));
                    } else {
                        unsigned w = 0u;
#pragma unroll
                        for (int e = 0; e < VEC; ++e)
                            w |= (c0 + e < d) ? (unsigned)p16[e] << (16 * e) : 0u;
                        raw[j] = w;
                    }
                    continue;
                }
                const float *p = G + (int64_t)r * ld + c0;
                if (VEC == 4 && full) {
                    const floatx4 v = __builtin_nontemporal_load(reinterpret_cast<const floatx4 *>(p));
                    x[j][0] = v[0]; x[j][1 % VEC] = v[1]; x[j][2 % VEC] = v[2]; x[j][3 % VEC] = v[3];
                } else if (VEC == 2 && full) {
                    const floatx2 v = __builtin_nontemporal_load(reinterpret_cast<const floatx2 *>(p));
                    x[j][0] = v[0]; x[j][1 % VEC] = v[1];
                } else {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) x[j][e] = (c0 + e < d) ? p[e] : 0.0f;
                }
            }
        }
        if constexpr (IN16) {
#pragma unroll
            for (int j = 0; j < kRows; ++j) {
                x[j][0] = widen16<IN16 ? FMT : kStoreBf16>(raw[j], false);
                x[j][1 % VEC] = widen16<IN16 ? FMT : kStoreBf16>(raw[j], VEC == 2);
            }
        }
#pragma unroll
        for (int j = 0; j < kRows; ++j)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] += x[j][e];
    }
    const float inv = m > 0 ? 1.0f / (float)m : 0.0f;
    if (full && VEC == 4 && ((uintptr_t)out % 16 == 0)) {
        const floatx4 o = {acc[0] * inv, acc[1 % VEC] * inv, acc[2 % VEC] * inv, acc[3 % VEC] * inv};
        __builtin_nontemporal_store(o, reinterpret_cast<floatx4 *>(out + c0));
        return;
    }
    if (full && VEC == 2 && ((uintptr_t)out % 8 == 0)) {
        const floatx2 o = {acc[0] * inv, acc[1 % VEC] * inv};
        __builtin_nontemporal_store(o, reinterpret_cast<floatx2 *>(out + c0));
        return;
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e)
        if (c0 + e < d) out[c0 + e] = acc[e] * inv;
}

// The plan from sets the caller supplies (coordwise_trimmed_avg with agr_sets); the aggregate entry
// points get theirs from select_kernel.
constexpr int kPlanThreads = 256;

__global__ __launch_bounds__(kPlanThreads) void alg1_plan_kernel(int n, int theta, const int32_t *__restrict__ sel,
                                                                 const uint8_t *__restrict__ sets,
                                                                 int32_t *__restrict__ plan)
{
    alg1_plan_body<kPlanThreads>(n, theta, sel, sets, plan, (int)threadIdx.x);
}

}  // namespace

hipError_t launch_alg1_plan(int n, int theta, const int32_t *sel, const uint8_t *sets, int32_t *plan,
                            hipStream_t s)
{
    alg1_plan_kernel<<<dim3(1), dim3(kPlanThreads), 0, s>>>(n, theta, sel, sets, plan);
    return hipGetLastError();
}

hipError_t launch_masked_mean(const float *G, int n, int64_t d, int64_t ld, const uint8_t *mask,
                              float *out, hipStream_t s)
{
    const bool aligned = ((uintptr_t)G % 16 == 0) && (ld % 4 == 0);
    if (aligned && d >= ((int64_t)1 << 24))
        masked_mean_kernel<2, kStoreFp32, kRowsLarge><<<dim3((unsigned)((d + 511) / 512)), dim3(256), 0, s>>>(G, n, d, ld, mask, out);
    else if (aligned)
        masked_mean_kernel<4, kStoreFp32, kRowsDefault><<<dim3((unsigned)((d + 1023) / 1024)), dim3(256), 0, s>>>(G, n, d, ld, mask, out);
    else
        masked_mean_kernel<1, kStoreFp32, kRowsDefault><<<dim3((unsigned)((d + 255) / 256)), dim3(256), 0, s>>>(G, n, d, ld, mask, out);
    return hipGetLastError();
}

hipError_t launch_masked_mean_in16(const uint16_t *G, int fmt, int n, int64_t d, int64_t ld, const uint8_t *mask,
                                   float *out, hipStream_t s)
{
    const bool aligned = ((uintptr_t)G % 4 == 0) && (ld % 2 == 0);
    const dim3 grid2((unsigned)((d + 511) / 512)), grid1((unsigned)((d + 255) / 256));
    if (fmt == kStoreBf16) {
        if (aligned) masked_mean_kernel<2, kStoreBf16, kRowsDefault><<<grid2, dim3(256), 0, s>>>(G, n, d, ld, mask, out);
        else masked_mean_kernel<1, kStoreBf16, kRowsDefault><<<grid1, dim3(256), 0, s>>>(G, n, d, ld, mask, out);
    } else if (fmt == kStoreFp16) {
        if (aligned) masked_mean_kernel<2, kStoreFp16, kRowsDefault><<<grid2, dim3(256), 0, s>>>(G, n, d, ld, mask, out);
        else masked_mean_kernel<1, kStoreFp16, kRowsDefault><<<grid1, dim3(256), 0, s>>>(G, n, d, ld, mask, out);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace mb
