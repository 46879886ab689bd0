/*
 * Host-side sanitizer run of the fp64 CPU oracle (TEST INFRASTRUCTURE, like the oracle itself):
 * compiled together with svgd_oracle.c under -fsanitize=address,undefined, this program drives
 * every oracle routine over small problems held in exactly-sized heap buffers - every shape class
 * the tests use (n = 1, n = 2, even and odd n, ragged D, column chunks that do not start at 0,
 * fp32 and fp64 inputs, fixed bandwidth, running moments) - so that an out-of-bounds access, a
 * misaligned or overflowing operation aborts the run.  It also re-checks a few closed forms
 * (paper App. B.2 in the score/ascent convention) so that the instrumented build is known to
 * compute the same thing.  Exit status 0 = clean.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void oracle_pairwise_d2(const void *X, int is_f64, int n, int64_t D, double *d2);
double oracle_median_all(const double *d2, int n);
double oracle_bandwidth(const double *d2, int n);
void oracle_kernel(const double *d2, int n, double h, double *K, double *r);
void oracle_phi_cols(const void *X, const void *G, int is_f64, int n, int64_t D, const double *K, double h,
                     int64_t col0, int64_t ncols, double *phi);
void oracle_step(const void *X, const void *G, int is_f64, int n, int64_t D, double eps, double h_fixed,
                 double *d2_out, double *K_out, double *r_out, double *h_out, double *phi_out, double *X_new);
void oracle_swag_update(double *mean, double *sq, const void *X, int is_f64, int64_t total, int64_t count);

static unsigned long long rng_state = 88172645463325252ull;
static double rnd(void) /* xorshift, uniform in (-1, 1) */
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}

static int failures = 0;
#define CHECK(cond, ...)                                                                            \
    do {                                                                                            \
        if (!(cond)) {                                                                              \
            fprintf(stderr, "sanitize_check: " __VA_ARGS__);                                        \
            fprintf(stderr, "\n");                                                                  \
            ++failures;                                                                             \
        }                                                                                           \
    } while (0)

static void one_shape(int n, int64_t D, int is_f64, double h_fixed)
{
    const size_t nd = (size_t)n * (size_t)D;
    void *X = malloc(nd * (is_f64 ? 8 : 4)), *G = malloc(nd * (is_f64 ? 8 : 4));
    for (size_t e = 0; e < nd; ++e) {
        if (is_f64) {
            ((double *)X)[e] = rnd();
            ((double *)G)[e] = rnd();
        } else {
            ((float *)X)[e] = (float)rnd();
            ((float *)G)[e] = (float)rnd();
        }
    }
    double *d2 = malloc((size_t)n * n * 8), *K = malloc((size_t)n * n * 8), *r = malloc((size_t)n * 8);
    double *phi = malloc(nd * 8), *xn = malloc(nd * 8), h = 0.0;
    oracle_step(X, G, is_f64, n, D, 0.1, h_fixed, d2, K, r, &h, phi, xn);
    CHECK(h > 0.0 && isfinite(h), "h = %g at n=%d D=%lld", h, n, (long long)D);
    for (int i = 0; i < n; ++i) {
        CHECK(K[(size_t)i * n + i] == 1.0 && d2[(size_t)i * n + i] == 0.0, "diagonal at n=%d", n);
        for (int j = 0; j < n; ++j) CHECK(K[(size_t)i * n + j] == K[(size_t)j * n + i], "K not symmetric at n=%d", n);
    }
    /* a chunk of columns that starts past 0 and ends at D agrees with the whole */
    if (D >= 3) {
        const int64_t c0 = D / 3, nc = D - c0;
        double *part = malloc((size_t)n * (size_t)nc * 8);
        oracle_phi_cols(X, G, is_f64, n, D, K, h, c0, nc, part);
        for (int i = 0; i < n; ++i)
            for (int64_t c = 0; c < nc; ++c)
                CHECK(part[(size_t)i * nc + c] == phi[(size_t)i * D + c0 + c], "phi chunk differs at n=%d D=%lld", n, (long long)D);
        free(part);
    }
    /* n = 1: plain gradient ascent, h = 1 */
    if (n == 1 && h_fixed <= 0.0) {
        CHECK(h == 1.0, "h = %g at n = 1", h);
        for (int64_t k = 0; k < D; ++k) {
            const double g = is_f64 ? ((double *)G)[k] : (double)((float *)G)[k];
            CHECK(fabs(phi[k] - g) <= 1e-15 * fabs(g), "phi != g at n = 1");
        }
    }
    /* n = 2: median of {0, 0, d, d} = d/2, so K_12 = exp(-2 ln 3) = 1/9 */
    if (n == 2 && h_fixed <= 0.0 && d2[1] > 0.0) CHECK(fabs(K[1] - 1.0 / 9.0) < 1e-14, "K12 = %.17g at n = 2", K[1]);
    /* the repulsive part sums to zero over the particles: sum_i [n phi_i - sum_j K_ij g_j] = 0 */
    for (int64_t k = 0; k < D; ++k) {
        double s = 0.0, scale = 0.0;
        for (int i = 0; i < n; ++i) {
            double kg = 0.0;
            for (int j = 0; j < n; ++j)
                kg += K[(size_t)i * n + j] * (is_f64 ? ((double *)G)[(size_t)j * D + k] : (double)((float *)G)[(size_t)j * D + k]);
            s += n * phi[(size_t)i * D + k] - kg;
            scale += fabs(n * phi[(size_t)i * D + k]) + fabs(kg);
        }
        CHECK(fabs(s) <= 1e-12 * (scale + 1.0), "repulsion does not cancel at n=%d column %lld: %g", n, (long long)k, s);
    }
    CHECK(oracle_median_all(d2, n) >= 0.0 && oracle_bandwidth(d2, n) > 0.0, "median / bandwidth at n=%d", n);
    free(X); free(G); free(d2); free(K); free(r); free(phi); free(xn);
}

int main(void)
{
    const int ns[] = {1, 2, 3, 4, 5, 8, 16, 17, 33, 64};
    const int64_t Ds[] = {1, 2, 3, 7, 64, 65, 257};
    for (unsigned a = 0; a < sizeof ns / sizeof *ns; ++a)
        for (unsigned b = 0; b < sizeof Ds / sizeof *Ds; ++b)
            for (int f64 = 0; f64 < 2; ++f64) {
                one_shape(ns[a], Ds[b], f64, 0.0);
                if (b % 3 == 0) one_shape(ns[a], Ds[b], f64, 2.5);
            }
    /* all particles equal: median 0 -> h = 1, K = 1 */
    {
        const int n = 5;
        const int64_t D = 9;
        float *X = malloc((size_t)n * D * 4), *G = malloc((size_t)n * D * 4);
        for (int i = 0; i < n; ++i)
            for (int64_t k = 0; k < D; ++k) {
                X[i * D + k] = (float)(0.25 * (double)k);
                G[i * D + k] = (float)rnd();
            }
        double h = 0.0, *K = malloc((size_t)n * n * 8);
        oracle_step(X, G, 0, n, D, 0.1, 0.0, NULL, K, NULL, &h, NULL, NULL);
        CHECK(h == 1.0, "coincident particles: h = %g", h);
        for (int e = 0; e < n * n; ++e) CHECK(K[e] == 1.0, "coincident particles: K = %g", K[e]);
        free(X); free(G); free(K);
    }
    /* running moments: three updates of a 3 x 5 matrix against the definition */
    {
        const int64_t total = 15;
        double *mean = calloc(total, 8), *sq = calloc(total, 8), sum[15] = {0}, sum2[15] = {0};
        float *x = malloc(total * 4);
        for (int t = 0; t < 3; ++t) {
            for (int e = 0; e < total; ++e) {
                x[e] = (float)rnd();
                sum[e] += x[e];
                sum2[e] += (double)x[e] * x[e];
            }
            oracle_swag_update(mean, sq, x, 0, total, t);
        }
        for (int e = 0; e < total; ++e)
            CHECK(fabs(mean[e] - sum[e] / 3) < 1e-15 && fabs(sq[e] - sum2[e] / 3) < 1e-15, "running moments, entry %d", e);
        free(mean); free(sq); free(x);
    }
    if (failures) {
        fprintf(stderr, "sanitize_check: %d failed checks\n", failures);
        return 1;
    }
    printf("sanitize_check: clean\n");
    return 0;
}
