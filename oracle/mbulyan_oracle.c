/*
 * CPU oracle for the multi-Bulyan gradient aggregation rule.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against.  It is used by the tests, by the smoke
 * check and by the CPU-baseline leg of the benchmark; the product path never
 * calls it and shares no code, header, table or helper with it.
 *
 * Everything is written from the paper (arxiv 1905.04374), Algorithm 1 and
 * Section II-B, step by step and in the paper's order:
 *   - squared l2 distances between all pairs of gradients (Algorithm 1,
 *     function multi-Krum, the score line; Eq. 4),
 *   - the Krum score of a gradient = sum of squared distances to its
 *     k-f-2 closest other gradients (Algorithm 1, multi-Krum; footnote 1 of
 *     Section I for the "-2"),
 *   - winner = smallest score, multi-Krum output = average of the m = k-f-2
 *     smallest scores (Algorithm 1, multi-Krum),
 *   - theta rounds of multi-Krum on the gradients not yet extracted
 *     (Algorithm 1, function multi-Bulyan, the loop),
 *   - coordinate-wise median, the beta values closest to it, their average
 *     (Algorithm 1, multi-Bulyan, after the loop; Section II-B last
 *     sentence on Bulyan).
 *
 * Arithmetic: inputs are fp32; every sum is accumulated in fp64, one term
 * after the other in the order the definition gives (coordinate 0..d-1,
 * neighbours in ascending distance).  No blocking, no reordering.  Threads
 * only split work whose items are independent (different pairs, different
 * coordinates), so the result does not depend on the thread count.
 *
 * Readings taken where the paper leaves a choice (each is listed with its
 * reason in the design notes of the repository):
 *   - two modes.  MODE_SELECTED follows the prose of Section II-B and the
 *     proof of Theorem 2(i): theta = n-2f rounds, and the median / beta
 *     closest / average run on the theta extracted gradients themselves.
 *     MODE_ALG1 follows Algorithm 1 to the letter: theta = n-2f-2, the
 *     median is taken over the extracted gradients G^ext and the beta
 *     closest values are taken among, and averaged over, the multi-Krum
 *     averages G^agr.  beta = theta-2f in both.
 *   - the loop of Algorithm 1 runs theta times (t = 0..theta-1); the printed
 *     upper bound would overflow the arrays the algorithm declares.
 *   - a gradient is not its own neighbour (footnote 1, Section I).
 *   - ties between scores: the smaller worker index first.
 *   - neighbour count max(k-f-2, 0).
 *   - even theta: median = 0.5*(lo+hi) of the two middle values, in fp32.
 *   - "closest to the median": the absolute difference is one fp32
 *     subtraction (the precision the values have), ties go to the smaller
 *     value (the earlier position in ascending order).
 *
 * parity pins: see tests/test_oracle_*.py (scipy pdist, brute force over
 * subsets, numpy mean / median, invariants).  No function here is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_MAX_N 1024

enum { ORC_MODE_SELECTED = 0, ORC_MODE_ALG1 = 1 };
enum { ORC_OK = 0, ORC_EINVAL = -1, ORC_EPRECOND = -2 };

/* Number of threads really used by the last threaded call (for reporting). */
static int g_last_threads = 1;
int orc_last_threads(void) { return g_last_threads; }

static int clamp_threads(int nthreads)
{
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
    return nthreads < 1 ? 1 : nthreads;
#else
    (void)nthreads;
    return 1;
#endif
}

/* Section II-B: multi-Bulyan needs n >= 4f+3.  theta and beta per mode. */
int orc_params(int n, int f, int mode, int *theta, int *beta)
{
    if (n < 1 || f < 0) return ORC_EINVAL;
    if (mode != ORC_MODE_SELECTED && mode != ORC_MODE_ALG1) return ORC_EINVAL;
    if (n < 4 * f + 3) return ORC_EPRECOND;
    int th = (mode == ORC_MODE_SELECTED) ? n - 2 * f : n - 2 * f - 2;
    int be = th - 2 * f;
    if (theta) *theta = th;
    if (beta) *beta = be;
    return ORC_OK;
}

/*
 * D[i][j] = sum over coordinates c of (G[i][c] - G[j][c])^2   (Algorithm 1,
 * the score line of multi-Krum; Eq. 4).  G is n rows of d floats, row i at
 * G + i*ld.  D is n*n doubles, row-major, symmetric, zero diagonal.
 * accumulate != 0 adds to what D holds (column chunks of one big matrix).
 */
void orc_pairwise_sqdist(const float *G, int n, int64_t d, int64_t ld,
                         double *D, int accumulate, int nthreads)
{
    int npairs = n * (n - 1) / 2;
    if (!accumulate)
        for (int i = 0; i < n * n; ++i) D[i] = 0.0;
    nthreads = clamp_threads(nthreads);
    g_last_threads = nthreads;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int p = 0; p < npairs; ++p) {
        /* p -> (i, j), i < j, in row order */
        int i = 0, rem = p;
        while (rem >= n - 1 - i) { rem -= n - 1 - i; ++i; }
        int j = i + 1 + rem;
        const float *a = G + (int64_t)i * ld;
        const float *b = G + (int64_t)j * ld;
        double s = 0.0;
        for (int64_t c = 0; c < d; ++c) {
            double diff = (double)a[c] - (double)b[c];
            s += diff * diff;
        }
        D[i * n + j] += s;
        D[j * n + i] += s;
    }
}

/* ascending insertion sort of doubles */
static void sort_doubles(double *v, int len)
{
    for (int a = 1; a < len; ++a) {
        double x = v[a];
        int b = a - 1;
        while (b >= 0 && v[b] > x) { v[b + 1] = v[b]; --b; }
        v[b + 1] = x;
    }
}

/*
 * Krum scores on the active set (Algorithm 1, multi-Krum): k = number of
 * active gradients, q = max(k-f-2, 0) neighbours; S[i] = sum of the q smallest
 * D[i][j] over active j != i, added in ascending order.  Inactive: +inf.
 * active == NULL means all active.
 */
void orc_krum_scores(const double *D, int n, int f, const uint8_t *active,
                     double *S)
{
    double row[ORC_MAX_N];
    int k = 0;
    for (int i = 0; i < n; ++i) k += (!active || active[i]) ? 1 : 0;
    int q = k - f - 2;
    if (q < 0) q = 0;
    for (int i = 0; i < n; ++i) {
        if (active && !active[i]) { S[i] = INFINITY; continue; }
        int len = 0;
        for (int j = 0; j < n; ++j) {
            if (j == i) continue;
            if (active && !active[j]) continue;
            row[len++] = D[i * n + j];
        }
        sort_doubles(row, len);
        double s = 0.0;
        for (int a = 0; a < q && a < len; ++a) s += row[a];
        S[i] = s;
    }
}

/*
 * theta rounds of multi-Krum on the gradients not yet extracted
 * (Algorithm 1, multi-Bulyan, the loop).  Round t works on the k = n-t
 * active gradients: scores with q = max(k-f-2,0); order the active gradients
 * by (score, index); ext[t] = the first; agr_sets[t][r] = 1 for the first
 * m_t = q of them (the gradients multi-Krum averages into G^agr[t]);
 * then ext[t] leaves the active set.
 * agr_sets (theta*n bytes), m_out (theta ints) and score_log (theta*n doubles,
 * the scores of every round, +inf for inactive) may be NULL.
 */
int orc_multikrum_select(const double *D, int n, int f, int theta,
                         int32_t *ext, uint8_t *agr_sets, int32_t *m_out,
                         double *score_log)
{
    if (n < 1 || n > ORC_MAX_N || f < 0 || theta < 0 || theta > n)
        return ORC_EINVAL;
    uint8_t active[ORC_MAX_N];
    double S[ORC_MAX_N];
    int order[ORC_MAX_N];
    for (int i = 0; i < n; ++i) active[i] = 1;
    for (int t = 0; t < theta; ++t) {
        int k = n - t;
        int q = k - f - 2;
        if (q < 0) q = 0;
        orc_krum_scores(D, n, f, active, S);
        if (score_log)
            for (int i = 0; i < n; ++i) score_log[t * n + i] = S[i];
        /* active indices ordered by (score, index): insertion sort */
        int len = 0;
        for (int i = 0; i < n; ++i) {
            if (!active[i]) continue;
            int b = len - 1;
            while (b >= 0 && S[order[b]] > S[i]) { order[b + 1] = order[b]; --b; }
            order[b + 1] = i; /* equal scores keep ascending index */
            ++len;
        }
        ext[t] = order[0];
        if (agr_sets) {
            for (int i = 0; i < n; ++i) agr_sets[t * n + i] = 0;
            for (int a = 0; a < q && a < len; ++a) agr_sets[t * n + order[a]] = 1;
        }
        if (m_out) m_out[t] = q < len ? q : len;
        active[order[0]] = 0;
    }
    return ORC_OK;
}

/* ascending insertion sort of floats */
static void sort_floats(float *v, int len)
{
    for (int a = 1; a < len; ++a) {
        float x = v[a];
        int b = a - 1;
        while (b >= 0 && v[b] > x) { v[b + 1] = v[b]; --b; }
        v[b + 1] = x;
    }
}

/* median of an ascending fp32 array: the middle value, or for an even count
 * the fp32 mean of the two middle values */
static float median_sorted(const float *v, int len)
{
    if (len & 1) return v[len / 2];
    volatile float s = v[len / 2 - 1] + v[len / 2];
    return 0.5f * s;
}

/*
 * From the ascending array v[0..len) pick the beta entries closest to med:
 * delta = |v - med| as one fp32 subtraction, order (delta, position).
 * Returns the fp64 sum of the picked entries added in ascending position,
 * and the fp64 sum of their absolute values in *abs_sum.
 */
static double pick_closest(const float *v, int len, float med, int beta,
                           double *abs_sum, uint8_t *picked)
{
    float delta[ORC_MAX_N];
    for (int p = 0; p < len; ++p) {
        volatile float df = v[p] - med;
        delta[p] = fabsf(df);
        picked[p] = 0;
    }
    for (int b = 0; b < beta; ++b) {
        int best = -1;
        for (int p = 0; p < len; ++p) {
            if (picked[p]) continue;
            if (best < 0 || delta[p] < delta[best]) best = p;
        }
        picked[best] = 1;
    }
    double s = 0.0, sa = 0.0;
    for (int p = 0; p < len; ++p)
        if (picked[p]) { s += (double)v[p]; sa += fabs((double)v[p]); }
    if (abs_sum) *abs_sum = sa;
    return s;
}

/*
 * Coordinate-wise phase, MODE_SELECTED (Section II-B, last sentence on
 * Bulyan; Theorem 2(i)): for every coordinate c take the theta values
 * G[ext[t]][c], their median, the beta values closest to it, their average.
 * out[c] = (float)(sum/beta).  scale (may be NULL) receives the mean absolute
 * value of the beta averaged values, the conditioning scale of out[c].
 */
void orc_coordwise_selected(const float *G, int64_t d, int64_t ld,
                            const int32_t *ext, int theta, int beta,
                            float *out, float *scale, int nthreads)
{
    nthreads = clamp_threads(nthreads);
    g_last_threads = nthreads;
#pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int64_t c = 0; c < d; ++c) {
        float v[ORC_MAX_N];
        uint8_t picked[ORC_MAX_N];
        for (int t = 0; t < theta; ++t) v[t] = G[(int64_t)ext[t] * ld + c];
        sort_floats(v, theta);
        float med = median_sorted(v, theta);
        double sa;
        double s = pick_closest(v, theta, med, beta, &sa, picked);
        out[c] = (float)(s / (double)beta);
        if (scale) scale[c] = (float)(sa / (double)beta);
    }
}

/*
 * Coordinate-wise phase, MODE_ALG1 (Algorithm 1, multi-Bulyan, after the
 * loop): M[c] = median over t of G^ext[t][c] = G[ext[t]][c];
 * G^agr[t][c] = average over the rows r with agr_sets[t][r] of G[r][c]
 * (fp64 sum in ascending r, divided by m_t, rounded to fp32: the precision
 * the method works in); out[c] = average of the beta values G^agr[.][c]
 * closest to M[c].
 * scale (may be NULL): the largest, over the rounds, of the mean absolute value
 * of the gradients averaged into G^agr[t][c]: the conditioning scale of an
 * fp32 evaluation of those averages.
 * margin (may be NULL): gap, in fp32, between the beta-th smallest |G^agr - M|
 * and the smallest one among the values not chosen that differ from the
 * beta-th value; alt (may be NULL): the output if that value replaced the
 * beta-th.  A comparison may accept alt where margin is below the rounding
 * noise of an fp32 evaluation of G^agr.
 */
void orc_coordwise_alg1(const float *G, int n, int64_t d, int64_t ld,
                        const int32_t *ext, const uint8_t *agr_sets,
                        int theta, int beta, float *out, float *scale,
                        float *margin, float *alt, int nthreads)
{
    nthreads = clamp_threads(nthreads);
    g_last_threads = nthreads;
#pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int64_t c = 0; c < d; ++c) {
        float e[ORC_MAX_N], a[ORC_MAX_N], delta[ORC_MAX_N];
        uint8_t picked[ORC_MAX_N];
        for (int t = 0; t < theta; ++t) e[t] = G[(int64_t)ext[t] * ld + c];
        sort_floats(e, theta);
        float med = median_sorted(e, theta);
        double cond = 0.0;
        for (int t = 0; t < theta; ++t) {
            double s = 0.0, sabs = 0.0;
            int m = 0;
            for (int r = 0; r < n; ++r)
                if (agr_sets[t * n + r]) {
                    s += (double)G[(int64_t)r * ld + c];
                    sabs += fabs((double)G[(int64_t)r * ld + c]);
                    ++m;
                }
            a[t] = (m > 0) ? (float)(s / (double)m) : 0.0f;
            if (m > 0 && sabs / (double)m > cond) cond = sabs / (double)m;
        }
        sort_floats(a, theta);
        double s = pick_closest(a, theta, med, beta, NULL, picked);
        out[c] = (float)(s / (double)beta);
        if (scale) scale[c] = (float)cond;
        if (margin || alt) {
            /* worst picked, by (delta, position), and the best not-picked value that differs
             * from it: swapping in an equal value would be no alternative at all (averages of
             * few-bit inputs repeat, and three-way ties do occur) */
            int worst = -1, next = -1;
            for (int p = 0; p < theta; ++p) {
                volatile float df = a[p] - med;
                delta[p] = fabsf(df);
            }
            for (int p = 0; p < theta; ++p)
                if (picked[p] && (worst < 0 || delta[p] >= delta[worst])) worst = p;
            for (int p = 0; p < theta; ++p)
                if (!picked[p] && a[p] != a[worst] && (next < 0 || delta[p] < delta[next])) next = p;
            if (next < 0) {
                if (margin) margin[c] = INFINITY;
                if (alt) alt[c] = out[c];
            } else {
                if (margin) margin[c] = delta[next] - delta[worst];
                if (alt) alt[c] = (float)((s - (double)a[worst] + (double)a[next]) / (double)beta);
            }
        }
    }
}

/*
 * Multi-Krum as a GAR of its own (Algorithm 1, function multi-Krum, the
 * returned G^output): average of the m = n-f-2 gradients of smallest score.
 * selected_mask (n bytes, may be NULL) receives the averaged set.
 */
int orc_multikrum_aggregate(const float *G, int n, int f, int64_t d,
                            int64_t ld, float *out, uint8_t *selected_mask,
                            int nthreads)
{
    if (n < 1 || n > ORC_MAX_N || f < 0) return ORC_EINVAL;
    if (n < 2 * f + 3) return ORC_EPRECOND;
    double *D = (double *)malloc(sizeof(double) * n * n);
    int32_t ext[1];
    uint8_t *sets = (uint8_t *)malloc((size_t)n);
    int32_t m[1];
    orc_pairwise_sqdist(G, n, d, ld, D, 0, nthreads);
    orc_multikrum_select(D, n, f, 1, ext, sets, m, NULL);
    nthreads = clamp_threads(nthreads);
#pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int64_t c = 0; c < d; ++c) {
        double s = 0.0;
        for (int r = 0; r < n; ++r)
            if (sets[r]) s += (double)G[(int64_t)r * ld + c];
        out[c] = (float)(s / (double)m[0]);
    }
    if (selected_mask) memcpy(selected_mask, sets, (size_t)n);
    free(D);
    free(sets);
    return ORC_OK;
}

/*
 * Coordinate-wise median of all n gradients (the Median GAR the paper
 * compares with, Section V): middle value, or fp32 mean of the two middle
 * values for even n.
 */
void orc_coordwise_median(const float *G, int n, int64_t d, int64_t ld,
                          float *out, int nthreads)
{
    nthreads = clamp_threads(nthreads);
#pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int64_t c = 0; c < d; ++c) {
        float v[ORC_MAX_N];
        for (int r = 0; r < n; ++r) v[r] = G[(int64_t)r * ld + c];
        sort_floats(v, n);
        out[c] = median_sorted(v, n);
    }
}

/*
 * GAR(f, [G_1..G_n]) = multi-Bulyan (Algorithm 1, function GAR).
 * ext receives the theta extracted indices in extraction order.
 * Returns ORC_OK, ORC_EINVAL or ORC_EPRECOND (n < 4f+3).
 */
int orc_mbulyan(const float *G, int n, int f, int64_t d, int64_t ld, int mode,
                float *out, int32_t *ext, int nthreads)
{
    int theta, beta;
    int rc = orc_params(n, f, mode, &theta, &beta);
    if (rc != ORC_OK) return rc;
    if (n > ORC_MAX_N || d < 1 || ld < d) return ORC_EINVAL;
    double *D = (double *)malloc(sizeof(double) * n * n);
    uint8_t *sets = (uint8_t *)malloc((size_t)theta * n + 1);
    int32_t *m = (int32_t *)malloc(sizeof(int32_t) * (theta + 1));
    int32_t *e = ext ? ext : (int32_t *)malloc(sizeof(int32_t) * (theta + 1));
    orc_pairwise_sqdist(G, n, d, ld, D, 0, nthreads);
    orc_multikrum_select(D, n, f, theta, e, sets, m, NULL);
    if (mode == ORC_MODE_SELECTED)
        orc_coordwise_selected(G, d, ld, e, theta, beta, out, NULL, nthreads);
    else
        orc_coordwise_alg1(G, n, d, ld, e, sets, theta, beta, out, NULL, NULL,
                           NULL, nthreads);
    if (!ext) free(e);
    free(m);
    free(sets);
    free(D);
    return ORC_OK;
}
