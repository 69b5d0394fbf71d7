/* Driver for the sanitizer build of the CPU oracle (tests/test_oracle_sanitizers.py compiles this
 * file together with oracle/mbulyan_oracle.c under -fsanitize=address,undefined and runs it).
 * It calls every entry point of the oracle on small inputs that reach the loop bounds: one
 * gradient, one coordinate, a row stride larger than d, theta = n, empty averaged sets, duplicate
 * rows, inactive gradients, both modes, several thread counts.  Results are not checked here (the
 * pin tests do that); any out-of-bounds access, misaligned access, signed overflow or leak ends
 * the process with a non-zero status. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int orc_params(int n, int f, int mode, int *theta, int *beta);
void orc_pairwise_sqdist(const float *G, int n, int64_t d, int64_t ld, double *D, int accumulate, int nthreads);
void orc_krum_scores(const double *D, int n, int f, const uint8_t *active, double *S);
int orc_multikrum_select(const double *D, int n, int f, int theta, int32_t *ext, uint8_t *agr_sets, int32_t *m_out,
                         double *score_log);
void orc_coordwise_selected(const float *G, int64_t d, int64_t ld, const int32_t *ext, int theta, int beta,
                            float *out, float *scale, int nthreads);
void orc_coordwise_alg1(const float *G, int n, int64_t d, int64_t ld, const int32_t *ext, const uint8_t *agr_sets,
                        int theta, int beta, float *out, float *scale, float *margin, float *alt, int nthreads);
int orc_multikrum_aggregate(const float *G, int n, int f, int64_t d, int64_t ld, float *out, uint8_t *selected_mask,
                            int nthreads);
void orc_coordwise_median(const float *G, int n, int64_t d, int64_t ld, float *out, int nthreads);
int orc_mbulyan(const float *G, int n, int f, int64_t d, int64_t ld, int mode, float *out, int32_t *ext, int nthreads);

static uint64_t state = 88172645463325252ull;
static float rnd(void)
{
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (float)((double)(state >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}

static void one_shape(int n, int f, int64_t d, int64_t ld, int threads)
{
    float *G = malloc(sizeof(float) * (size_t)n * (size_t)ld);
    for (int64_t i = 0; i < (int64_t)n * ld; ++i) G[i] = rnd();
    if (n >= 3) for (int64_t c = 0; c < d; ++c) G[(int64_t)(n - 1) * ld + c] = G[c];      /* a duplicate row */
    double *D = malloc(sizeof(double) * (size_t)n * n);
    orc_pairwise_sqdist(G, n, d, ld, D, 0, threads);
    orc_pairwise_sqdist(G, n, d > 1 ? d / 2 : d, ld, D, 1, threads);                       /* accumulate a chunk */
    double *S = malloc(sizeof(double) * (size_t)n);
    uint8_t *active = malloc((size_t)n);
    for (int i = 0; i < n; ++i) active[i] = (uint8_t)(i % 3 != 1);
    orc_krum_scores(D, n, f, NULL, S);
    orc_krum_scores(D, n, f, active, S);
    for (int theta = 1; theta <= n; theta += (n > 4 ? n / 4 : 1)) {
        int32_t *ext = malloc(sizeof(int32_t) * (size_t)theta);
        uint8_t *sets = malloc((size_t)theta * (size_t)n);
        int32_t *m = malloc(sizeof(int32_t) * (size_t)theta);
        double *log = malloc(sizeof(double) * (size_t)theta * (size_t)n);
        if (orc_multikrum_select(D, n, f, theta, ext, sets, m, log) != 0) exit(3);
        orc_multikrum_select(D, n, f, theta, ext, NULL, NULL, NULL);
        float *out = malloc(sizeof(float) * (size_t)d), *scale = malloc(sizeof(float) * (size_t)d);
        float *margin = malloc(sizeof(float) * (size_t)d), *alt = malloc(sizeof(float) * (size_t)d);
        for (int beta = 1; beta <= theta; beta += (theta > 3 ? theta / 3 : 1)) {
            orc_coordwise_selected(G, d, ld, ext, theta, beta, out, scale, threads);
            orc_coordwise_selected(G, d, ld, ext, theta, beta, out, NULL, threads);
            orc_coordwise_alg1(G, n, d, ld, ext, sets, theta, beta, out, scale, margin, alt, threads);
            orc_coordwise_alg1(G, n, d, ld, ext, sets, theta, beta, out, NULL, NULL, NULL, threads);
        }
        free(out); free(scale); free(margin); free(alt); free(ext); free(sets); free(m); free(log);
    }
    float *out = malloc(sizeof(float) * (size_t)d);
    int32_t *ext = malloc(sizeof(int32_t) * (size_t)n);
    uint8_t *mask = malloc((size_t)n);
    orc_coordwise_median(G, n, d, ld, out, threads);
    orc_multikrum_aggregate(G, n, f, d, ld, out, mask, threads);
    orc_multikrum_aggregate(G, n, f, d, ld, out, NULL, threads);
    for (int mode = 0; mode < 2; ++mode) {
        int theta = 0, beta = 0;
        if (orc_params(n, f, mode, &theta, &beta) == 0) {
            if (orc_mbulyan(G, n, f, d, ld, mode, out, ext, threads) != 0) exit(4);
            if (orc_mbulyan(G, n, f, d, ld, mode, out, NULL, threads) != 0) exit(4);
        } else if (orc_mbulyan(G, n, f, d, ld, mode, out, ext, threads) == 0) {
            exit(5);                                   /* the precondition must be refused */
        }
    }
    free(out); free(ext); free(mask); free(G); free(D); free(S); free(active);
}

int main(void)
{
    static const int shapes[][3] = {   /* n, f, d */
        {1, 0, 1}, {1, 0, 7}, {2, 0, 1}, {3, 0, 5}, {4, 0, 3}, {7, 1, 33}, {8, 1, 2}, {11, 2, 100},
        {11, 3, 9}, {19, 4, 257}, {39, 9, 64}, {64, 15, 17}, {64, 0, 3}};
    for (unsigned s = 0; s < sizeof(shapes) / sizeof(shapes[0]); ++s)
        for (int threads = 1; threads <= 4; threads += 3) {
            one_shape(shapes[s][0], shapes[s][1], shapes[s][2], shapes[s][2], threads);
            one_shape(shapes[s][0], shapes[s][1], shapes[s][2], shapes[s][2] + 5, threads);
        }
    puts("oracle sanitizer run: ok");
    return 0;
}
