/*
 * fp64 CPU oracle for one SVGD all-particle update (Liu & Wang's method as used
 * by the paper's App. B.2 "SVGD in Push" routine), written out from the
 * definition.  TEST INFRASTRUCTURE ONLY: it is slow on purpose, shares no code
 * with the GPU library, and nothing on the product path may call it.
 *
 * Notation (paper App. B.2): n particles, particle i is the flattened parameter
 * vector x_i of length D (row i of X), g_i = grad log p(x_i) (row i of G).
 *
 *   d2_ij  = sum_k (x_ik - x_jk)^2                      squared distance, direct differences
 *   med    = median of all n*n entries of d2            (diagonal zeros included; even count ->
 *                                                        mean of the two middle order statistics)
 *   h      = med / ln(n+1)                              median-heuristic bandwidth; h<=0 -> h=1
 *   K_ij   = exp(-d2_ij / h)                            RBF kernel; with h = 2*l^2 this is the
 *                                                        paper's exp(-|x_j-x_i|^2/(2 l^2))
 *   phi_ik = (1/n) sum_j [ K_ij g_jk + (2/h) K_ij (x_ik - x_jk) ]    j runs over ALL particles
 *   x_ik  <- x_ik + eps * phi_ik                        every phi from the pre-step X (Jacobi)
 *
 * Inputs may be fp32 or fp64 arrays (flag is_f64); all arithmetic is fp64.
 * Loops over columns carry plain OpenMP pragmas; nothing is blocked, fused or
 * reordered beyond that.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline double ld(const void *p, int is_f64, int64_t idx)
{
    return is_f64 ? ((const double *)p)[idx] : (double)((const float *)p)[idx];
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* d2 (n*n, row-major) from direct per-pair differences; diagonal exactly 0; mirrored. */
void oracle_pairwise_d2(const void *X, int is_f64, int n, int64_t D, double *d2)
{
    for (int i = 0; i < n; ++i) {
        d2[(int64_t)i * n + i] = 0.0;
        for (int j = i + 1; j < n; ++j) {
            double s = 0.0;
#pragma omp parallel for reduction(+ : s) schedule(static)
            for (int64_t k = 0; k < D; ++k) {
                double diff = ld(X, is_f64, (int64_t)i * D + k) - ld(X, is_f64, (int64_t)j * D + k);
                s += diff * diff;
            }
            d2[(int64_t)i * n + j] = s;
            d2[(int64_t)j * n + i] = s;
        }
    }
}

static int cmp_double(const void *a, const void *b)
{
    double x = *(const double *)a, y = *(const double *)b;
    return (x > y) - (x < y);
}

/* Median of the multiset of all n*n entries of d2. */
double oracle_median_all(const double *d2, int n)
{
    int64_t m = (int64_t)n * n;
    double *tmp = (double *)malloc((size_t)m * sizeof(double));
    memcpy(tmp, d2, (size_t)m * sizeof(double));
    qsort(tmp, (size_t)m, sizeof(double), cmp_double);
    double med = (m % 2) ? tmp[m / 2] : 0.5 * (tmp[m / 2 - 1] + tmp[m / 2]);
    free(tmp);
    return med;
}

/* h = med(d2)/ln(n+1); a non-positive (or NaN) value is replaced by 1. */
double oracle_bandwidth(const double *d2, int n)
{
    double h = oracle_median_all(d2, n) / log((double)n + 1.0);
    if (!(h > 0.0)) h = 1.0;
    return h;
}

/* K_ij = exp(-d2_ij/h), r_i = sum_j K_ij. */
void oracle_kernel(const double *d2, int n, double h, double *K, double *r)
{
    for (int i = 0; i < n; ++i) {
        double s = 0.0;
        for (int j = 0; j < n; ++j) {
            double k = exp(-d2[(int64_t)i * n + j] / h);
            K[(int64_t)i * n + j] = k;
            s += k;
        }
        r[i] = s;
    }
}

/*
 * phi for columns [col0, col0+ncols), written to phi (n x ncols, row-major, fp64),
 * in the per-pair difference form: phi_ik = (1/n) sum_j K_ij [ g_jk + (2/h)(x_ik - x_jk) ].
 */
void oracle_phi_cols(const void *X, const void *G, int is_f64, int n, int64_t D,
                     const double *K, double h, int64_t col0, int64_t ncols, double *phi)
{
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < ncols; ++c) {
        int64_t k = col0 + c;
        for (int i = 0; i < n; ++i) {
            double xi = ld(X, is_f64, (int64_t)i * D + k);
            double acc = 0.0;
            for (int j = 0; j < n; ++j) {
                double kij = K[(int64_t)i * n + j];
                double gj = ld(G, is_f64, (int64_t)j * D + k);
                double xj = ld(X, is_f64, (int64_t)j * D + k);
                acc += kij * gj + (2.0 / h) * kij * (xi - xj);
            }
            phi[(int64_t)i * ncols + c] = acc / (double)n;
        }
    }
}

/*
 * One whole step.  Outputs (any may be NULL): d2, K (n*n), r (n), h_out (1),
 * phi (n*D fp64), X_new (n*D fp64) = X + eps*phi.  If h_fixed > 0 it is used
 * in place of the median heuristic (the paper's fixed lengthscale l maps to
 * h = 2 l^2).
 */
void oracle_step(const void *X, const void *G, int is_f64, int n, int64_t D, double eps,
                 double h_fixed, double *d2_out, double *K_out, double *r_out, double *h_out,
                 double *phi_out, double *X_new)
{
    double *d2 = (double *)malloc((size_t)n * n * sizeof(double));
    double *K = (double *)malloc((size_t)n * n * sizeof(double));
    double *r = (double *)malloc((size_t)n * sizeof(double));
    oracle_pairwise_d2(X, is_f64, n, D, d2);
    double h = (h_fixed > 0.0) ? h_fixed : oracle_bandwidth(d2, n);
    oracle_kernel(d2, n, h, K, r);
    if (phi_out || X_new) {
        double *phi = phi_out ? phi_out : (double *)malloc((size_t)n * D * sizeof(double));
        oracle_phi_cols(X, G, is_f64, n, D, K, h, 0, D, phi);
        if (X_new) {
            for (int64_t e = 0; e < (int64_t)n * D; ++e) X_new[e] = ld(X, is_f64, e) + eps * phi[e];
        }
        if (!phi_out) free(phi);
    }
    if (d2_out) memcpy(d2_out, d2, (size_t)n * n * sizeof(double));
    if (K_out) memcpy(K_out, K, (size_t)n * n * sizeof(double));
    if (r_out) memcpy(r_out, r, (size_t)n * sizeof(double));
    if (h_out) *h_out = h;
    free(d2);
    free(K);
    free(r);
}

/*
 * SWAG / multi-SWAG running moments (paper Sec. 2: SWAG keeps the first and second moments of a
 * network's parameter trajectory; multi-SWAG does so for every particle of an ensemble).
 * After `count` earlier updates the running means absorb one more iterate x (the published SWAG
 * recursion of Maddox et al.):
 *     mean <- (count * mean + x) / (count + 1),    sq <- (count * sq + x^2) / (count + 1)
 * for every entry of the n x D particle matrix.  mean and sq are fp64 arrays updated in place.
 */
void oracle_swag_update(double *mean, double *sq, const void *X, int is_f64, int64_t total, int64_t count)
{
    const double c = (double)count;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < total; ++e) {
        double x = ld(X, is_f64, e);
        mean[e] = (c * mean[e] + x) / (c + 1.0);
        sq[e] = (c * sq[e] + x * x) / (c + 1.0);
    }
}
