// multi-Bulyan over gradients that stay in host memory (d beyond what the device holds: Section I speaks
// of d up to 10^9 .. 10^11): column chunks are uploaded into two device buffers in turn, the upload of
// chunk c+1 overlapping the kernels of chunk c.
//
// Two sweeps over the host matrix are inherent: the selection needs the distances over all
// coordinates (Algorithm 1 computes them over whole gradients) before any coordinate can be
// aggregated.  Sweep 1: upload, distance pass accumulating into one n x n matrix.  Then the
// selection.  Sweep 2: upload again, coordinate pass, download of that chunk's part of the result.
// A matrix that fits the device next to everything else is uploaded once instead: sweep 1 leaves the
// chunks in one device matrix and the coordinate pass runs over it in one go (half the bytes over
// the link).  "Fits": n d values within mbulyan_host_resident_limit (default: three quarters of the
// device memory that is free when the call starts; 0 switches the single upload off).
// Everything the kernels do goes through the library's own entry points (pairwise_sqdist with
// accumulate, multikrum_select, coordwise_trimmed_avg); this file only moves data and orders events.
// Copies run on a stream of their own (default priority), kernels on the caller's stream.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>

#include "../../include/mbulyan.h"

namespace {

std::atomic<long long> g_resident_limit{-1};   // bytes; -1: three quarters of the free device memory
constexpr int kTwoSweepsInstead = -1000;        // internal: the device matrix could not be allocated after all

struct Guard {   // frees what the call allocated, whatever way it ends
    void *dev[8] = {};
    int ndev = 0;
    hipStream_t copy = nullptr;
    hipStream_t compute = nullptr;
    bool launched = false;
    hipEvent_t ev[6] = {};
    int nev = 0;
    ~Guard()
    {
        // nothing of this call may still be running when its buffers go (also on an error path)
        if (copy) (void)hipStreamSynchronize(copy);
        if (launched) (void)hipStreamSynchronize(compute);
        for (int i = 0; i < nev; ++i) (void)hipEventDestroy(ev[i]);
        if (copy) (void)hipStreamDestroy(copy);
        for (int i = 0; i < ndev; ++i) (void)hipFree(dev[i]);
    }
    hipError_t alloc(void **p, size_t bytes)
    {
        const hipError_t e = hipMalloc(p, bytes);
        if (e == hipSuccess) dev[ndev++] = *p;
        return e;
    }
    hipError_t event(hipEvent_t *e)
    {
        const hipError_t rc = hipEventCreateWithFlags(e, hipEventDisableTiming);
        if (rc == hipSuccess) ev[nev++] = *e;
        return rc;
    }
};

#define HC_HIP(expr)                              \
    do {                                          \
        if ((expr) != hipSuccess) return MB_EHIP; \
    } while (0)
#define HC_MB(expr)               \
    do {                          \
        const int rc_ = (expr);   \
        if (rc_ != MB_OK) return rc_; \
    } while (0)

int dist_chunk(const void *buf, int storage, int n, int64_t w, double *dist, int accumulate, void *ws, size_t ws_bytes,
               hipStream_t s)
{
    switch (storage) {
        case MB_STORE_FP32:
            return pairwise_sqdist(static_cast<const float *>(buf), n, w, w, dist, accumulate, MB_DIST_AUTO, ws, ws_bytes, s);
        case MB_STORE_BF16:
            return pairwise_sqdist_bf16(static_cast<const uint16_t *>(buf), n, w, w, dist, accumulate, ws, ws_bytes, s);
        default:
            return pairwise_sqdist_fp16(static_cast<const uint16_t *>(buf), n, w, w, dist, accumulate, ws, ws_bytes, s);
    }
}

int coord_chunk(const void *buf, int storage, int n, int64_t w, int64_t ld, const int32_t *sel, int theta, int beta,
                const uint8_t *sets, float *out, hipStream_t s)
{
    switch (storage) {
        case MB_STORE_FP32:
            return coordwise_trimmed_avg(static_cast<const float *>(buf), n, w, ld, sel, theta, beta, sets, out, s);
        case MB_STORE_BF16:
            return coordwise_trimmed_avg_bf16(static_cast<const uint16_t *>(buf), n, w, ld, sel, theta, beta, sets, out, s);
        default:
            return coordwise_trimmed_avg_fp16(static_cast<const uint16_t *>(buf), n, w, ld, sel, theta, beta, sets, out, s);
    }
}


// d small enough for the device: chunks are uploaded into one n x d device matrix (row stride d)
// while the distance pass follows them chunk by chunk; the coordinate pass then takes the whole
// matrix at once.
int aggregate_uploaded_once(const void *host_grads, int storage, int n, int f, int64_t d, int64_t ld, int mode,
                            int64_t chunk_d, int theta, int beta, float *host_out, int32_t *host_selected_idx,
                            hipStream_t compute)
{
    const size_t eb = storage == MB_STORE_FP32 ? 4 : 2;
    // chunks start on 16-byte boundaries of the device rows (the fast load path of the distance pass)
    const int64_t per16 = (int64_t)(16 / eb);
    if (chunk_d % per16) chunk_d += per16 - chunk_d % per16;
    const int64_t nchunks = (d + chunk_d - 1) / chunk_d;
    const int64_t ldd = (d + per16 - 1) / per16 * per16;   // device rows start on 16-byte boundaries as well
    Guard g;
    g.compute = compute;
    size_t ws_bytes = 0;
    HC_MB(mbulyan_workspace_bytes(n, d, &ws_bytes));
    void *whole = nullptr, *ws = nullptr;
    double *dist = nullptr;
    float *out = nullptr;
    int32_t *sel = nullptr;
    uint8_t *sets = nullptr;
    if (g.alloc(&whole, eb * (size_t)n * (size_t)ldd) != hipSuccess) {   // free memory, but not in one piece
        (void)hipGetLastError();
        return kTwoSweepsInstead;
    }
    HC_HIP(g.alloc(&ws, ws_bytes));
    HC_HIP(g.alloc(reinterpret_cast<void **>(&dist), sizeof(double) * (size_t)n * n));
    HC_HIP(g.alloc(reinterpret_cast<void **>(&out), sizeof(float) * (size_t)d));
    HC_HIP(g.alloc(reinterpret_cast<void **>(&sel), 2 * sizeof(int32_t) * (size_t)theta));
    HC_HIP(g.alloc(reinterpret_cast<void **>(&sets), (size_t)theta * (size_t)n));
    int32_t *m = sel + theta;
    HC_HIP(hipStreamCreateWithFlags(&g.copy, hipStreamNonBlocking));   // default priority
    hipEvent_t start, uploaded[2];
    HC_HIP(g.event(&start));
    HC_HIP(g.event(&uploaded[0]));
    HC_HIP(g.event(&uploaded[1]));
    g.launched = true;
    HC_HIP(hipEventRecord(start, compute));      // the caller's earlier work on its stream comes first
    HC_HIP(hipStreamWaitEvent(g.copy, start, 0));
    const char *src = static_cast<const char *>(host_grads);
    char *dst = static_cast<char *>(whole);
    for (int64_t c = 0; c < nchunks; ++c) {
        const int64_t c0 = c * chunk_d, w = (c0 + chunk_d <= d) ? chunk_d : d - c0;
        const int k = (int)(c & 1);
        HC_HIP(hipMemcpy2DAsync(dst + eb * (size_t)c0, eb * (size_t)ldd, src + eb * (size_t)c0, eb * (size_t)ld,
                                eb * (size_t)w, (size_t)n, hipMemcpyHostToDevice, g.copy));
        // an event may be recorded again once the wait on its last record has been enqueued: two in turn
        HC_HIP(hipEventRecord(uploaded[k], g.copy));
        HC_HIP(hipStreamWaitEvent(compute, uploaded[k], 0));
        const void *chunk = dst + eb * (size_t)c0;
        switch (storage) {
            case MB_STORE_FP32:
                HC_MB(pairwise_sqdist(static_cast<const float *>(chunk), n, w, ldd, dist, c > 0, MB_DIST_AUTO, ws, ws_bytes,
                                      compute));
                break;
            case MB_STORE_BF16:
                HC_MB(pairwise_sqdist_bf16(static_cast<const uint16_t *>(chunk), n, w, ldd, dist, c > 0, ws, ws_bytes,
                                           compute));
                break;
            default:
                HC_MB(pairwise_sqdist_fp16(static_cast<const uint16_t *>(chunk), n, w, ldd, dist, c > 0, ws, ws_bytes,
                                           compute));
        }
    }
    HC_MB(multikrum_select(dist, n, f, theta, sel, sets, m, compute));
    HC_MB(coord_chunk(whole, storage, n, d, ldd, sel, theta, beta, mode == MB_MODE_ALG1 ? sets : nullptr, out, compute));
    HC_HIP(hipMemcpyAsync(host_out, out, sizeof(float) * (size_t)d, hipMemcpyDeviceToHost, compute));
    if (host_selected_idx)
        HC_HIP(hipMemcpyAsync(host_selected_idx, sel, sizeof(int32_t) * (size_t)theta, hipMemcpyDeviceToHost, compute));
    HC_HIP(hipStreamSynchronize(g.copy));
    HC_HIP(hipStreamSynchronize(compute));
    return MB_OK;
}

}  // namespace

extern "C" int mbulyan_host_resident_limit(long long bytes)
{
    g_resident_limit.store(bytes < 0 ? -1 : bytes);
    return MB_OK;
}

extern "C" int mbulyan_aggregate_host(const void *host_grads, int storage, int n, int f, int64_t d, int64_t ld, int mode,
                                      int64_t chunk_d, float *host_out, int32_t *host_selected_idx, void *stream)
{
    if (!host_grads || !host_out || n < 1 || d < 1 || ld < d || f < 0 || chunk_d < 1) return MB_EINVAL;
    if (storage != MB_STORE_FP32 && storage != MB_STORE_BF16 && storage != MB_STORE_FP16) return MB_EINVAL;
    int theta = 0, beta = 0;
    HC_MB(mbulyan_params(n, f, mode, &theta, &beta));   // MB_EPRECOND / MB_EUNSUPPORTED / MB_EINVAL
    if (chunk_d > d) chunk_d = d;
    const size_t eb = storage == MB_STORE_FP32 ? 4 : 2;
    const int64_t nchunks = (d + chunk_d - 1) / chunk_d;
    hipStream_t compute = (hipStream_t)stream;

    // the whole matrix on the device, if it fits: one upload
    {
        long long limit = g_resident_limit.load();
        if (limit < 0) {
            size_t free_b = 0, total_b = 0;
            HC_HIP(hipMemGetInfo(&free_b, &total_b));
            limit = (long long)(free_b / 4 * 3);
        }
        size_t whole_ws = 0;
        HC_MB(mbulyan_workspace_bytes(n, d, &whole_ws));
        const double need = (double)eb * n * ((double)d + 8.0) + 4.0 * (double)d + (double)whole_ws + 65536.0;
        if (need <= (double)limit) {
            const int rc = aggregate_uploaded_once(host_grads, storage, n, f, d, ld, mode, chunk_d, theta, beta, host_out,
                                                   host_selected_idx, compute);
            if (rc != kTwoSweepsInstead) return rc;
        }
    }

    Guard g;
    g.compute = compute;
    size_t ws_bytes = 0;
    HC_MB(mbulyan_workspace_bytes(n, chunk_d, &ws_bytes));
    void *buf[2] = {}, *ws = nullptr;
    double *dist = nullptr;
    float *out[2] = {};
    int32_t *sel = nullptr;
    uint8_t *sets = nullptr;
    HC_HIP(g.alloc(&buf[0], eb * (size_t)n * (size_t)chunk_d));
    HC_HIP(g.alloc(&buf[1], eb * (size_t)n * (size_t)chunk_d));
    HC_HIP(g.alloc(&ws, ws_bytes));
    HC_HIP(g.alloc(reinterpret_cast<void **>(&dist), sizeof(double) * (size_t)n * n));
    HC_HIP(g.alloc(reinterpret_cast<void **>(&out[0]), sizeof(float) * (size_t)chunk_d));
    HC_HIP(g.alloc(reinterpret_cast<void **>(&out[1]), sizeof(float) * (size_t)chunk_d));
    HC_HIP(g.alloc(reinterpret_cast<void **>(&sel), sizeof(int32_t) * (size_t)theta + sizeof(int32_t) * (size_t)theta));
    HC_HIP(g.alloc(reinterpret_cast<void **>(&sets), (size_t)theta * (size_t)n));
    int32_t *m = sel + theta;
    HC_HIP(hipStreamCreateWithFlags(&g.copy, hipStreamNonBlocking));   // default priority
    hipEvent_t uploaded[2], consumed[2], produced[2];
    for (int k = 0; k < 2; ++k) {
        HC_HIP(g.event(&uploaded[k]));
        HC_HIP(g.event(&consumed[k]));
        HC_HIP(g.event(&produced[k]));
    }
    // the caller's earlier work on its stream comes first (the host matrix may be its product)
    hipEvent_t start = uploaded[0];
    g.launched = true;
    HC_HIP(hipEventRecord(start, compute));
    HC_HIP(hipStreamWaitEvent(g.copy, start, 0));

    const char *src = static_cast<const char *>(host_grads);
    auto upload = [&](int64_t c, int k) -> hipError_t {
        const int64_t c0 = c * chunk_d, w = (c0 + chunk_d <= d) ? chunk_d : d - c0;
        // n rows of w values: host row stride ld, device rows packed (stride w)
        return hipMemcpy2DAsync(buf[k], eb * (size_t)w, src + eb * (size_t)c0, eb * (size_t)ld, eb * (size_t)w, (size_t)n,
                                hipMemcpyHostToDevice, g.copy);
    };

    bool used[2] = {false, false};   // consumed[k] has been recorded: kernels may still be reading buffer k
    bool wrote[2] = {false, false};  // produced[k] has been recorded: a download of out[k] may be pending
    for (int sweep = 0; sweep < 2; ++sweep) {
        for (int64_t c = 0; c < nchunks; ++c) {
            const int k = (int)(c & 1);
            const int64_t c0 = c * chunk_d, w = (c0 + chunk_d <= d) ? chunk_d : d - c0;
            if (used[k]) HC_HIP(hipStreamWaitEvent(g.copy, consumed[k], 0));   // the kernels of chunk c-2 are done with it
            HC_HIP(upload(c, k));
            HC_HIP(hipEventRecord(uploaded[k], g.copy));
            HC_HIP(hipStreamWaitEvent(compute, uploaded[k], 0));
            if (sweep == 0) {
                HC_MB(dist_chunk(buf[k], storage, n, w, dist, c > 0, ws, ws_bytes, compute));
            } else {
                if (wrote[k]) HC_HIP(hipStreamWaitEvent(compute, produced[k], 0));   // out[k] has been downloaded
                HC_MB(coord_chunk(buf[k], storage, n, w, w, sel, theta, beta, mode == MB_MODE_ALG1 ? sets : nullptr, out[k],
                                  compute));
            }
            HC_HIP(hipEventRecord(consumed[k], compute));
            used[k] = true;
            if (sweep == 1) {
                HC_HIP(hipStreamWaitEvent(g.copy, consumed[k], 0));
                HC_HIP(hipMemcpyAsync(host_out + c0, out[k], sizeof(float) * (size_t)w, hipMemcpyDeviceToHost, g.copy));
                HC_HIP(hipEventRecord(produced[k], g.copy));
                wrote[k] = true;
            }
        }
        if (sweep == 0) {
            HC_MB(multikrum_select(dist, n, f, theta, sel, sets, m, compute));
            // the second sweep's uploads may start at once: they only need their buffers, which the
            // loop above orders through consumed[]
        }
    }
    if (host_selected_idx) {
        HC_HIP(hipMemcpyAsync(host_selected_idx, sel, sizeof(int32_t) * (size_t)theta, hipMemcpyDeviceToHost, compute));
    }
    // the buffers are this call's own: it cannot return before everything that uses them is done
    HC_HIP(hipStreamSynchronize(g.copy));
    HC_HIP(hipStreamSynchronize(compute));
    return MB_OK;
}
