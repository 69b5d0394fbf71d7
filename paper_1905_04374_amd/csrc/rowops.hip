// Row averages: the multi-Krum output G^output = average of the m gradients of
// smallest score (Algorithm 1, function multi-Krum).  One lane owns four
// consecutive coordinates (one when the matrix is not 16-byte aligned) and
// adds the selected rows in ascending row order; the membership mask is
// uniform, so rows outside the set are skipped without being read.
#include <hip/hip_runtime.h>

#include "mb_internal.hpp"

namespace mb {
namespace {

template <int VEC>
__global__ __launch_bounds__(256) void masked_mean_kernel(const float *__restrict__ G, int n, int64_t d,
                                                          int64_t ld, const uint8_t *__restrict__ mask,
                                                          float *__restrict__ out)
{
    const int64_t c0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * VEC;
    if (c0 >= d) return;
    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.0f;
    int m = 0;
    const bool full = c0 + VEC <= d;
    for (int r = 0; r < n; ++r) {
        if (!mask[r]) continue;
        ++m;
        const float *p = G + (int64_t)r * ld + c0;
        if (VEC == 4 && full) {
            const float4 x = *reinterpret_cast<const float4 *>(p);
            acc[0] += x.x; acc[1] += x.y; acc[2] += x.z; acc[3] += x.w;
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] += (c0 + e < d) ? p[e] : 0.0f;
        }
    }
    const float inv = m > 0 ? 1.0f / (float)m : 0.0f;
#pragma unroll
    for (int e = 0; e < VEC; ++e)
        if (c0 + e < d) out[c0 + e] = acc[e] * inv;
}

}  // namespace

hipError_t launch_masked_mean(const float *G, int n, int64_t d, int64_t ld, const uint8_t *mask,
                              float *out, hipStream_t s)
{
    const bool aligned = ((uintptr_t)G % 16 == 0) && (ld % 4 == 0);
    if (aligned)
        masked_mean_kernel<4><<<dim3((unsigned)((d + 1023) / 1024)), dim3(256), 0, s>>>(G, n, d, ld, mask, out);
    else
        masked_mean_kernel<1><<<dim3((unsigned)((d + 255) / 256)), dim3(256), 0, s>>>(G, n, d, ld, mask, out);
    return hipGetLastError();
}

}  // namespace mb
