/*
 * SD-KDE reference oracle: TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, double-precision CPU implementation of the three steps of the SD-KDE
 * pipeline, written directly from the definitions in the paper.  It exists to check the
 * GPU library and to be timed as a CPU baseline; nothing in the product path may call it.
 * It shares no code with the GPU path: it forms every pairwise difference explicitly and
 * never uses the Gram-matrix expansion of the squared distance nor the Phi*X regrouping of
 * the score numerator.
 *
 * All arrays are host memory, row-major, contiguous, doubles.  OpenMP parallelises over
 * evaluation points only; each point's sums run over the samples in index order.
 * Return value 0 on success, 1 on invalid arguments, 2 on allocation failure.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int sdkde_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* a_j = -||p - x_j||^2 / (2 h^2): the exponent of the Gaussian kernel (Method section,
 * definition of phi_ij), by direct differences.  Returns max_j a_j. */
static double exponents(const double *X, int64_t n, int32_t d, const double *p, double h,
                        double *a)
{
    double amax = -INFINITY;
    for (int64_t j = 0; j < n; ++j) {
        const double *xj = X + j * (int64_t)d;
        double r2 = 0.0;
        for (int32_t k = 0; k < d; ++k) {
            double diff = p[k] - xj[k];
            r2 += diff * diff;
        }
        a[j] = -r2 / (2.0 * h * h);
        if (a[j] > amax) amax = a[j];
    }
    return amax;
}

/*
 * Empirical score (Introduction, the displayed formula for s-hat):
 *   s(p) = sum_j -(p - x_j) phi_j / (h^2 sum_j phi_j),  phi_j = exp(-||p - x_j||^2 / 2h^2).
 * The kernel's normalising constant cancels between numerator and denominator.  Every
 * weight is divided by the largest one, exp(amax), which also cancels and only keeps far
 * points from underflowing.  The sum runs over all n samples, so when p is itself a sample
 * its own term is included (numerator 0, denominator 1).
 * X: samples [n,d]; P: evaluation points [m,d]; S: out [m,d].
 */
int sdkde_oracle_score(const double *X, int64_t n, const double *P, int64_t m, int32_t d,
                       double h, double *S)
{
    if (!X || !P || !S || n < 1 || m < 0 || d < 1 || !(h > 0.0) || !isfinite(h)) return 1;
    int fail = 0;
#pragma omp parallel
    {
        double *a = (double *)malloc(sizeof(double) * (size_t)n);
        double *num = (double *)malloc(sizeof(double) * (size_t)d);
        if (!a || !num) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 16)
            for (int64_t i = 0; i < m; ++i) {
                const double *p = P + i * (int64_t)d;
                double amax = exponents(X, n, d, p, h, a);
                double den = 0.0;
                for (int32_t k = 0; k < d; ++k) num[k] = 0.0;
                for (int64_t j = 0; j < n; ++j) {
                    const double *xj = X + j * (int64_t)d;
                    double w = exp(a[j] - amax);
                    den += w;
                    for (int32_t k = 0; k < d; ++k) num[k] += -(p[k] - xj[k]) * w;
                }
                for (int32_t k = 0; k < d; ++k) S[i * (int64_t)d + k] = num[k] / (h * h * den);
            }
        }
        free(a);
        free(num);
    }
    return fail ? 2 : 0;
}

/* Debiasing shift (Introduction): x_sd = x + (h^2 / 2) s(x).  Elementwise over [n,d]. */
int sdkde_oracle_debias(const double *X, const double *S, int64_t n, int32_t d, double h,
                        double *Xsd)
{
    if (!X || !S || !Xsd || n < 0 || d < 1 || !(h > 0.0) || !isfinite(h)) return 1;
    int64_t total = n * (int64_t)d;
    for (int64_t t = 0; t < total; ++t) Xsd[t] = X[t] + 0.5 * h * h * S[t];
    return 0;
}

/*
 * Gaussian KDE (Introduction, first display; normalised kernel K_h of the Laplace-corrected
 * KDE section):
 *   p(q) = 1/(n h^d) sum_j phi((q - x_j)/h),  phi(u) = (2 pi)^(-d/2) exp(-||u||^2 / 2).
 * Evaluated in log space: log p = amax + log sum_j exp(a_j - amax) - log n - d log h
 * - (d/2) log(2 pi).  Either output pointer may be NULL.
 * laplace == 1 multiplies each term by (1 + d/2 - ||q - x_j||^2 / 2h^2), the
 * Laplace-corrected kernel K_h^LC; the sum can then be negative, so only `dens` is
 * written (logdens must be NULL).  laplace == 2 uses the absolute value of that factor:
 * the magnitude against which the rounding of the signed sum is judged.
 * Xs: samples [n,d]; Q: queries [m,d]; logdens, dens: out [m].
 */
static int eval_impl(const double *Xs, int64_t n, const double *Q, int64_t m, int32_t d,
                     double h, double *logdens, double *dens, int laplace)
{
    if (!Xs || !Q || (!logdens && !dens) || n < 1 || m < 0 || d < 1 || !(h > 0.0) ||
        !isfinite(h))
        return 1;
    if (laplace && logdens) return 1;
    const double two_pi = 6.283185307179586476925286766559;
    const double lognorm = -log((double)n) - (double)d * log(h) - 0.5 * (double)d * log(two_pi);
    int fail = 0;
#pragma omp parallel
    {
        double *a = (double *)malloc(sizeof(double) * (size_t)n);
        if (!a) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 16)
            for (int64_t i = 0; i < m; ++i) {
                double amax = exponents(Xs, n, d, Q + i * (int64_t)d, h, a);
                double sum = 0.0;
                if (!laplace) {
                    for (int64_t j = 0; j < n; ++j) sum += exp(a[j] - amax);
                    double lp = amax + log(sum) + lognorm;
                    if (logdens) logdens[i] = lp;
                    if (dens) dens[i] = exp(lp);
                } else {
                    /* a_j = -r^2/2h^2, so the affine factor is 1 + d/2 + a_j */
                    for (int64_t j = 0; j < n; ++j) {
                        double factor = 1.0 + 0.5 * (double)d + a[j];
                        if (laplace == 2) factor = fabs(factor);
                        sum += exp(a[j] - amax) * factor;
                    }
                    dens[i] = sum * exp(amax + lognorm);
                }
            }
        }
        free(a);
    }
    return fail ? 2 : 0;
}

int sdkde_oracle_eval(const double *Xs, int64_t n, const double *Q, int64_t m, int32_t d,
                      double h, double *logdens, double *dens)
{
    return eval_impl(Xs, n, Q, m, d, h, logdens, dens, 0);
}

/* Laplace-corrected KDE (Laplace-corrected KDE section): p_LC(q) = (1/n) sum_j K_h^LC(q - x_j). */
int sdkde_oracle_eval_laplace(const double *X, int64_t n, const double *Q, int64_t m, int32_t d,
                              double h, double *dens)
{
    return eval_impl(X, n, Q, m, d, h, NULL, dens, 1);
}

/* Same sum with |1 + d/2 - r^2/2h^2| in place of the signed factor (a tolerance scale, not an estimator). */
int sdkde_oracle_eval_laplace_abs(const double *X, int64_t n, const double *Q, int64_t m, int32_t d,
                                  double h, double *dens)
{
    return eval_impl(X, n, Q, m, d, h, NULL, dens, 2);
}
