/*
 * mbulyan.h - C ABI of the MI355X (gfx950) multi-Bulyan library.
 *
 * multi-Bulyan is the gradient aggregation rule (GAR) of "Fast and Robust
 * Distributed Learning in High Dimension" (arxiv 1905.04374), Algorithm 1:
 * given n worker gradients of dimension d, at most f of them Byzantine, it
 * runs theta rounds of multi-Krum on the pairwise squared distances, then,
 * per coordinate, averages the beta values closest to a median.
 *
 * Conventions shared by every entry point
 *   - Plain C, no exceptions.  Every call returns an MB_* status code.
 *   - Pointers marked "device" are GPU global memory owned by the caller
 *     (allocate them with anything that yields a HIP device pointer, e.g.
 *     PyTorch); the library neither frees nor keeps them.  Pointers marked
 *     "host" are ordinary process memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue their kernels on it and return without synchronising;
 *     outputs are valid once the caller has synchronised the stream.
 *   - Gradients: n rows of d floats (fp32), row i starting at grads + i*ld,
 *     ld >= d the row stride in elements.  Fastest when grads is 16-byte
 *     aligned and ld is a multiple of 4; other strides are handled by a
 *     slower load path.  Results are defined for finite inputs; a gradient
 *     that holds a NaN or an infinity is at distance +inf from every other,
 *     so it is never a neighbour and, while no more than f rows are like
 *     that, never chosen nor read by the coordinate pass.
 *   - n <= MB_MAX_N.
 *   - Arguments are validated on the host before anything is launched; an
 *     invalid call launches nothing.
 *   - Calls that share a workspace (or the internal one) must not overlap.
 *     Host threads may call concurrently with workspaces of their own; the
 *     internal workspace is one per device and is shared by every call that
 *     passes none.  It is allocated by the first such call on a device and
 *     reallocated when a later call needs more; such a call synchronises the
 *     device and allocates (so it cannot be captured into a HIP graph, and it
 *     is not "enqueue and return").  Callers who need neither pass a workspace
 *     of mbulyan_workspace_bytes(n, d) bytes or call mbulyan_aggregate_noalloc.
 *     mbulyan_aggregate_host is the one call that blocks by design.
 */
#ifndef MBULYAN_H
#define MBULYAN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MB_MAX_N 64

/* status codes */
#define MB_OK 0
#define MB_EINVAL 1       /* null pointer, n < 1, d < 1, ld < d, f < 0, bad mode / theta / beta */
#define MB_EPRECOND 2     /* n < 4f+3 (multi-Bulyan) or n < 2f+3 (multi-Krum); Section II-B */
#define MB_EUNSUPPORTED 3 /* n > MB_MAX_N */
#define MB_EWORKSPACE 4   /* workspace too small or misaligned (256 bytes) */
#define MB_EHIP 5         /* a HIP call failed; see mbulyan_last_hip_error() */

/*
 * The paper states the rule in two ways that differ; both are provided.
 * MB_MODE_SELECTED: Section II-B (last sentence on Bulyan) and the proof of
 *   Theorem 2(i): theta = n-2f rounds; median, beta closest and average are
 *   taken over the theta extracted gradients.  beta = theta-2f = n-4f.
 * MB_MODE_ALG1: Algorithm 1 as printed: theta = n-2f-2; the median is that
 *   of the extracted gradients G^ext, the beta closest values are chosen
 *   among, and averaged over, the multi-Krum averages G^agr.
 *   beta = theta-2f = n-4f-2.
 */
#define MB_MODE_SELECTED 0
#define MB_MODE_ALG1 1

/* how pairwise_sqdist evaluates the distances */
#define MB_DIST_AUTO 0   /* library picks */
#define MB_DIST_DIRECT 1 /* sum of (x_i - x_j)^2 on the vector ALU, fp32 partial sums */
#define MB_DIST_GRAM 2   /* Gram matrix on the fp32 matrix cores (MFMA), fp64 running sums,
                            D_ij = G_ii + G_jj - 2 G_ij in fp64.  The error of that form grows with
                            the norms, not with D_ij: where some pair has G_ii + G_jj > 256 D_ij
                            (gradients with a large common component) a second pass repeats the
                            Gram matrix on the rows minus a pivot row chosen among the bulk of
                            them, and every pair takes the better-conditioned of its two values */
#define MB_DIST_GRAM_BF16 3 /* the same Gram matrix on the bf16 matrix cores: every fp32 value is
                            split exactly into three bf16 pieces and the six significant piece
                            products are accumulated in fp32 (error of the order of one fp32
                            rounding per product) */

const char *mbulyan_strerror(int status);
/* hipError_t (as int) of the last failing HIP call on this thread, 0 if none */
int mbulyan_last_hip_error(void);
const char *mbulyan_version(void);

/*
 * theta and beta of a mode (table above).  Host only.
 * MB_EPRECOND if n < 4f+3 (Section II-B), MB_EINVAL for f < 0, n < 1 or an
 * unknown mode, MB_EUNSUPPORTED if n > MB_MAX_N.
 */
int mbulyan_params(int n, int f, int mode, int *theta, int *beta);

/*
 * Bytes of device workspace that pairwise_sqdist and mbulyan_aggregate_ex need
 * for n gradients of dimension d (per call, or per chunk for the chunked use).
 * The workspace must be 256-byte aligned device memory.  Host only.
 */
int mbulyan_workspace_bytes(int n, int64_t d, size_t *bytes);

/* Pick the distance algorithm used by MB_DIST_AUTO callers (process-wide; MB_DIST_AUTO restores
 * the default choice).  Host only. */
int mbulyan_set_dist_algo(int algo);

/*
 * GAR(f, [G_1..G_n]) = multi-Bulyan (Algorithm 1, function GAR), in
 * MB_MODE_SELECTED, ld = d.
 *   grads        device, n*d floats
 *   out          device, d floats: the aggregated gradient
 *   selected_idx device, n-2f int32 (may be NULL): the extracted workers in
 *                extraction order
 * Uses a workspace owned by the library (allocated on the first call on a
 * device and grown when a later call needs more; freed by mbulyan_release).
 * Launches: distance pass, its reduction, the second distance pass (returns at
 * once unless the first was ill conditioned), selection, coordinate pass.
 */
int mbulyan_aggregate(const float *grads, int n, int f, int64_t d, float *out,
                      int32_t *selected_idx, void *stream);

/*
 * As mbulyan_aggregate with everything explicit.
 *   mode          MB_MODE_SELECTED / MB_MODE_ALG1
 *   theta, beta   0 = the mode's default; otherwise 1 <= beta <= theta <= n
 *   workspace     device, ws_bytes >= mbulyan_workspace_bytes(n, d); NULL =
 *                 the library's own
 */
int mbulyan_aggregate_ex(const float *grads, int n, int f, int64_t d,
                         int64_t ld, int mode, int theta, int beta, float *out,
                         int32_t *selected_idx, void *workspace,
                         size_t ws_bytes, void *stream);

/*
 * mbulyan_aggregate_ex for callers that cannot allocate device memory or let
 * the library do it: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same kernels, same results; the workspace
 * is a device array of MB_NOALLOC_SCRATCH_BYTES that is part of the library
 * itself (every GPU the library runs on holds it until the process ends), so
 * the call allocates and frees nothing, on the device or through any library.
 * theta and beta are the mode's defaults.
 *   grads, out, selected_idx   as for mbulyan_aggregate_ex (selected_idx may
 *                              be NULL)
 * Limits: n <= MB_MAX_N (MB_EUNSUPPORTED beyond, nothing launched), any d: the
 * distance pass is launched with no more workgroups than the array has room
 * for (16 MiB hold the partial sums of at least 814 of them at n = 64, more
 * than stay resident on the device).  MB_EWORKSPACE if the array could not
 * hold one workgroup's sums (cannot happen with the sizes above).
 * The first call on a device looks up the address of that device's copy of the
 * array (the HIP runtime places the library's device variables at that point);
 * no later call touches the allocator.
 * All calls on one GPU share that GPU's array, which keeps the contents of the
 * last call (nothing in it has to start at zero: every stage reads only what
 * the stage before it wrote in the same call): calls that overlap on one GPU (different streams or threads)
 * race and must be serialised by the caller.  Per-stage timing
 * (mbulyan_timing_enable) does not see these calls.
 */
#define MB_NOALLOC_SCRATCH_BYTES (16u << 20)
int mbulyan_aggregate_noalloc(const float *grads, int n, int f, int64_t d,
                              int64_t ld, int mode, float *out,
                              int32_t *selected_idx, void *stream);

/*
 * The same rule over a matrix given as column chunks (for d too large for one
 * buffer): chunk c holds columns [sum of chunk_d[0..c), +chunk_d[c]) as n rows
 * of stride chunk_ld[c], and its part of the result goes to outs[c].
 * Distances are accumulated over all chunks first (Algorithm 1 computes them
 * over whole gradients), then one selection, then the coordinate pass per
 * chunk.
 *   chunks, outs      host arrays of nchunks device pointers
 *   chunk_d, chunk_ld host arrays of nchunks sizes
 */
int mbulyan_aggregate_chunked(const float *const *chunks, int nchunks,
                              const int64_t *chunk_d, const int64_t *chunk_ld,
                              int n, int f, int mode, float *const *outs,
                              int32_t *selected_idx, void *workspace,
                              size_t ws_bytes, void *stream);

/*
 * Pairwise squared l2 distances (Algorithm 1, multi-Krum, the score line;
 * Eq. 4): dist[i*n+j] = sum_c (G[i][c]-G[j][c])^2, symmetric, zero diagonal.
 *   dist       device, n*n doubles
 *   accumulate 0: overwrite dist; 1: add this call's distances to it (column
 *              chunks of one matrix)
 *   algo       MB_DIST_*
 * Bit-identical rows get bit-identical distance rows and distance exactly 0
 * to each other; the result does not depend on timing (no atomics).
 */
int pairwise_sqdist(const float *grads, int n, int64_t d, int64_t ld,
                    double *dist, int accumulate, int algo, void *workspace,
                    size_t ws_bytes, void *stream);

/*
 * Krum scores (Algorithm 1, multi-Krum; Eq. 4; footnote 1 of Section I):
 * with k active gradients and q = max(k-f-2, 0), scores[i] = sum of the q
 * smallest dist[i][j] over active j != i, added in ascending order in fp64.
 * Inactive gradients get +inf.
 *   dist   device, n*n doubles      active device, n bytes, NULL = all active
 *   scores device, n doubles
 */
int krum_scores(const double *dist, int n, int f, const uint8_t *active,
                double *scores, void *stream);

/*
 * theta rounds of multi-Krum on the gradients not yet extracted (Algorithm 1,
 * multi-Bulyan, the loop).  Round t: scores on the n-t active gradients;
 * order them by (score, index); selected_idx[t] = the first, which then
 * leaves the active set; agr_sets[t*n+r] = 1 for the first m_t =
 * max(n-t-f-2, 0) of them (the set multi-Krum averages), else 0.
 *   selected_idx device, theta int32
 *   agr_sets     device, theta*n bytes, may be NULL
 *   m_out        device, theta int32, may be NULL
 * Needs 1 <= theta <= n.  No precondition on (n, f) is imposed here.
 */
int multikrum_select(const double *dist, int n, int f, int theta,
                     int32_t *selected_idx, uint8_t *agr_sets, int32_t *m_out,
                     void *stream);

/*
 * Coordinate-wise phase (Algorithm 1, multi-Bulyan, after the loop; Section
 * II-B).  For every coordinate c:
 *   agr_sets == NULL: v_t = G[selected_idx[t]][c]; med = median of the v_t;
 *     out[c] = average of the beta values v_t closest to med.
 *   agr_sets != NULL: med = median over t of G[selected_idx[t]][c];
 *     a_t = average of G[r][c] over the rows r with agr_sets[t*n+r] != 0;
 *     out[c] = average of the beta values a_t closest to med.
 * Median of an even count: 0.5*(lo+hi) in fp32.  Closeness: |v-med| as one
 * fp32 subtraction; on equal closeness the smaller value is preferred.
 *   selected_idx device, theta int32 in [0, n), validated on the device: an
 *                out-of-range index makes the kernel write NaN to out, and so
 *                does, with agr_sets != NULL, an index that occurs twice
 *   out          device, d floats
 * With agr_sets != NULL an 18 KB plan is kept in the library's own workspace
 * (allocated on the first such call on a device; calls that use it must not
 * overlap on one device).
 */
int coordwise_trimmed_avg(const float *grads, int n, int64_t d, int64_t ld,
                          const int32_t *selected_idx, int theta, int beta,
                          const uint8_t *agr_sets, float *out, void *stream);

/*
 * Gradients stored in 16 bits (NEXT to the fp32 path: the same operations of
 * Algorithm 1 on half the bytes).  Two formats, raw 16-bit words, ld in
 * elements:
 *   *_bf16  bfloat16: the upper half of the fp32 bit pattern
 *   *_fp16  IEEE half precision (subnormals included)
 * Every value of either format is an fp32 value, so the results are those of
 * the fp32 entry points on the widened matrix, to the same tolerances;
 * distances and out stay fp64 / fp32.  The distance pass needs no splitting:
 * a product of two such values is exact in fp32 (one matrix-core product per
 * pair and coordinate); its second, centred pass works on the fp32
 * differences.  The fast paths need rows that start on 16-byte boundaries
 * (distance pass: grads % 16 == 0 and ld % 8 == 0) and 4-byte boundaries
 * (coordinate pass: grads % 4 == 0, ld % 2 == 0, out % 8 == 0); anything else
 * takes element loads.  Arguments as for the fp32 entry point of the same
 * name:
 *   pairwise_sqdist_*            pairwise_sqdist (Gram form)
 *   coordwise_trimmed_avg_*      coordwise_trimmed_avg
 *   mbulyan_aggregate_*          mbulyan_aggregate_ex
 *   mbulyan_aggregate_chunked_*  mbulyan_aggregate_chunked
 *   multikrum_aggregate_*        multikrum_aggregate
 *   coordwise_median_*           coordwise_median
 */
int pairwise_sqdist_bf16(const uint16_t *grads, int n, int64_t d, int64_t ld,
                         double *dist, int accumulate, void *workspace,
                         size_t ws_bytes, void *stream);
int coordwise_trimmed_avg_bf16(const uint16_t *grads, int n, int64_t d,
                               int64_t ld, const int32_t *selected_idx,
                               int theta, int beta, const uint8_t *agr_sets,
                               float *out, void *stream);
int mbulyan_aggregate_bf16(const uint16_t *grads, int n, int f, int64_t d,
                           int64_t ld, int mode, int theta, int beta,
                           float *out, int32_t *selected_idx, void *workspace,
                           size_t ws_bytes, void *stream);
int multikrum_aggregate_bf16(const uint16_t *grads, int n, int f, int64_t d,
                             int64_t ld, float *out, uint8_t *selected_mask,
                             void *workspace, size_t ws_bytes, void *stream);
int coordwise_median_bf16(const uint16_t *grads, int n, int64_t d, int64_t ld,
                          float *out, void *stream);
int mbulyan_aggregate_chunked_bf16(const uint16_t *const *chunks, int nchunks,
                                   const int64_t *chunk_d,
                                   const int64_t *chunk_ld, int n, int f,
                                   int mode, float *const *outs,
                                   int32_t *selected_idx,
                                   void *workspace, size_t ws_bytes,
                                   void *stream);
int pairwise_sqdist_fp16(const uint16_t *grads, int n, int64_t d, int64_t ld,
                         double *dist, int accumulate, void *workspace,
                         size_t ws_bytes, void *stream);
int coordwise_trimmed_avg_fp16(const uint16_t *grads, int n, int64_t d,
                               int64_t ld, const int32_t *selected_idx,
                               int theta, int beta, const uint8_t *agr_sets,
                               float *out, void *stream);
int mbulyan_aggregate_fp16(const uint16_t *grads, int n, int f, int64_t d,
                           int64_t ld, int mode, int theta, int beta,
                           float *out, int32_t *selected_idx, void *workspace,
                           size_t ws_bytes, void *stream);
int multikrum_aggregate_fp16(const uint16_t *grads, int n, int f, int64_t d,
                             int64_t ld, float *out, uint8_t *selected_mask,
                             void *workspace, size_t ws_bytes, void *stream);
int coordwise_median_fp16(const uint16_t *grads, int n, int64_t d, int64_t ld,
                          float *out, void *stream);
int mbulyan_aggregate_chunked_fp16(const uint16_t *const *chunks, int nchunks,
                                   const int64_t *chunk_d,
                                   const int64_t *chunk_ld, int n, int f,
                                   int mode, float *const *outs,
                                   int32_t *selected_idx,
                                   void *workspace, size_t ws_bytes,
                                   void *stream);

/*
 * The same rule for gradients that stay in HOST memory (d beyond what the device
 * holds; Section I speaks of d up to 10^9 .. 10^11).  Column chunks of chunk_d
 * coordinates are uploaded into two device buffers in turn, the upload of one
 * chunk overlapping the kernels of the one before, in two sweeps over the
 * matrix: distances (Algorithm 1 computes them over whole gradients), then the
 * selection, then the coordinate pass per chunk with its part of the result
 * copied back.
 *   host_grads   host, n rows of d values, row stride ld elements; pinned memory
 *                (hipHostMalloc) if the copies are to overlap the kernels,
 *                pageable memory works but serialises them
 *   storage      MB_STORE_FP32 (float), MB_STORE_BF16 / MB_STORE_FP16 (16-bit words)
 *   chunk_d      coordinates per chunk (the last chunk may be shorter); the call
 *                holds 2 n chunk_d values plus 2 chunk_d floats of device memory
 *   host_out     host, d floats
 *   host_selected_idx  host, theta int32, may be NULL
 *   stream       the kernels' stream (copies use a stream of the call's own); work
 *                queued on it before the call is waited for
 * theta and beta are the mode's defaults.  Unlike the other entry points this one
 * allocates and frees device memory (its chunk buffers) and RETURNS ONLY WHEN THE
 * RESULT IS IN host_out.  The rate is that of the host link, twice over: the
 * device-resident entry points are the ones to time.
 * A matrix that fits the device is uploaded once instead: the first sweep leaves
 * its chunks in one device matrix (n d values plus d floats and a workspace, for
 * the length of the call) and the coordinate pass runs over it in one go.  It
 * "fits" if that is within mbulyan_host_resident_limit: by default three quarters
 * of the device memory free when the call starts; 0 = always two sweeps; any
 * other value = that many bytes; negative = the default again.  Process-wide,
 * host only.  Same results either way.
 */
#define MB_STORE_FP32 0
#define MB_STORE_BF16 1
#define MB_STORE_FP16 2
int mbulyan_host_resident_limit(long long bytes);
int mbulyan_aggregate_host(const void *host_grads, int storage, int n, int f,
                           int64_t d, int64_t ld, int mode, int64_t chunk_d,
                           float *host_out, int32_t *host_selected_idx,
                           void *stream);

/*
 * Multi-Krum as a GAR (Algorithm 1, function multi-Krum, G^output): the
 * average of the m = n-f-2 gradients of smallest score.  Needs n >= 2f+3.
 *   selected_mask device, n bytes, may be NULL: 1 for the averaged gradients
 */
int multikrum_aggregate(const float *grads, int n, int f, int64_t d,
                        int64_t ld, float *out, uint8_t *selected_mask,
                        void *workspace, size_t ws_bytes, void *stream);

/*
 * Coordinate-wise median of all n gradients (the Median GAR the paper compares
 * with in Section V).
 */
int coordwise_median(const float *grads, int n, int64_t d, int64_t ld,
                     float *out, void *stream);

/*
 * Per-kernel timing of the calls above, with HIP events recorded on the call's
 * own stream.  mbulyan_timing_enable(stages) starts collecting for the stages
 * whose bits (1 << MB_STAGE_x) are set, MB_STAGE_ALL for all of them; (0)
 * stops.  Every timed stage puts two event records into the stream per call,
 * a few microseconds each: time one stage alone where a call takes less than
 * a millisecond.
 * mbulyan_timing_read synchronises the recorded events and returns, per stage,
 * the summed milliseconds and the number of launches since the last
 * mbulyan_timing_reset.  Stages: 0 distance pass (first pass of the Gram
 * forms), 1 distance reduction, 2 selection, 3 coordinate pass, 4 the second
 * pass of the Gram forms (launched every time; a few microseconds when the
 * first pass was well conditioned; it reduces its own partial sums).  Both arrays have
 * MB_NUM_STAGES entries.  Host only; not thread safe.
 */
#define MB_STAGE_DIST 0
#define MB_STAGE_REDUCE 1
#define MB_STAGE_SELECT 2
#define MB_STAGE_COORD 3
#define MB_STAGE_REFINE 4
#define MB_NUM_STAGES 5
#define MB_STAGE_ALL ((1 << MB_NUM_STAGES) - 1)
int mbulyan_timing_enable(int stages);
int mbulyan_timing_reset(void);
int mbulyan_timing_read(double *ms_per_stage, int64_t *launches_per_stage);

/* Free the library's own workspaces and timing events (all devices). */
int mbulyan_release(void);

#ifdef __cplusplus
}
#endif
#endif /* MBULYAN_H */
