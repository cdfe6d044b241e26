/*
 * lnmod_oracle.c -- float64 CPU oracle for the fused LayerNorm-Modulate (AdaLN) operator.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU path is
 * checked against.  It shares no code, header, table or helper with the HIP library and is
 * never called from the product path; only the tests, the smoke check and the benchmark's
 * "cpu_baseline" leg may load it.
 *
 * What it computes (paper Sec. 3.3 describes the operator in prose: per-token mean and
 * variance over the hidden dimension D, normalisation, then the modulation by shift/scale;
 * the backward pass yields dx and the modulation gradients reduced along the token axis):
 *
 *   mu_n    = (1/D) sum_d x[n,d]
 *   var_n   = (1/D) sum_d (x[n,d] - mu_n)^2          two passes, biased (divide by D)
 *   r_n     = 1 / sqrt(var_n + eps)
 *   xhat    = (x[n,d] - mu_n) * r_n
 *   y[n,d]  = xhat * (1 + scale[m,d]) + shift[m,d]   LayerNorm without affine, then modulate
 *
 *   g[n,d]  = dy[n,d] * (1 + scale[m,d])
 *   c1_n    = (1/D) sum_d g[n,d]
 *   c2_n    = (1/D) sum_d g[n,d] * xhat[n,d]
 *   dx[n,d] = r_n * (g[n,d] - c1_n - xhat[n,d] * c2_n)
 *   dshift[m,d] = sum_{n in m} dy[n,d]
 *   dscale[m,d] = sum_{n in m} dy[n,d] * xhat[n,d]
 *
 * m is the modulation row that token n uses: the segment that contains n (a sample of a
 * fixed-length batch is a segment of length S), or n itself in per-token mode, where the
 * "sums" have one term.  The backward recomputes mu and r itself; it never sees statistics
 * saved by anybody else.  Sums over tokens run in index order.
 *
 * Inputs arrive either as double or as float (in_f32 != 0).  A float input is only a carrier:
 * bf16 and fp32 values are exactly representable in it, and every operation below is done
 * in double.  Nothing here is blocked, fused or reordered beyond what the formulas state;
 * OpenMP only distributes independent token rows (and, for the token sums, independent
 * feature ranges) over threads, which does not change any result.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define LNMOD_ORACLE_PER_SEGMENT 0
#define LNMOD_ORACLE_PER_TOKEN 1

static inline double ld(const void *p, int in_f32, int64_t i)
{
    return in_f32 ? (double)((const float *)p)[i] : ((const double *)p)[i];
}

int lnmod_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void lnmod_oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* mean and reciprocal standard deviation of one row (two passes) */
static void row_stats(const void *x, int in_f32, int64_t row, int64_t D, double eps,
                      double *mu_out, double *r_out)
{
    double s = 0.0;
    for (int64_t d = 0; d < D; ++d) s += ld(x, in_f32, row * D + d);
    double mu = s / (double)D;
    double q = 0.0;
    for (int64_t d = 0; d < D; ++d) {
        double c = ld(x, in_f32, row * D + d) - mu;
        q += c * c;
    }
    double var = q / (double)D;
    *mu_out = mu;
    *r_out = 1.0 / sqrt(var + eps);
}

/*
 * Forward.  x [T,D]; cu [nseg+1] token offsets of the segments (cu[0]=0, cu[nseg]=T);
 * shift, scale [nseg,D] (mod = per segment) or [T,D] (mod = per token);
 * y [T,D], mean [T], rstd [T] in double.  Returns 0, or 1 for bad arguments.
 */
int lnmod_oracle_forward(const void *x, const void *shift, const void *scale, int in_f32,
                         const int64_t *cu, int64_t nseg, int64_t D, double eps, int mod,
                         double *y, double *mean, double *rstd)
{
    if (!cu || nseg < 0 || D <= 0) return 1;
    if (mod != LNMOD_ORACLE_PER_SEGMENT && mod != LNMOD_ORACLE_PER_TOKEN) return 1;
    for (int64_t m = 0; m < nseg; ++m)
        if (cu[m] < 0 || cu[m + 1] < cu[m]) return 1;       /* before anything is written */
    for (int64_t m = 0; m < nseg; ++m) {
        const int64_t n0 = cu[m], n1 = cu[m + 1];
#pragma omp parallel for schedule(static)
        for (int64_t n = n0; n < n1; ++n) {
            double mu, r;
            row_stats(x, in_f32, n, D, eps, &mu, &r);
            const int64_t mrow = (mod == LNMOD_ORACLE_PER_TOKEN) ? n : m;
            for (int64_t d = 0; d < D; ++d) {
                double xhat = (ld(x, in_f32, n * D + d) - mu) * r;
                y[n * D + d] = xhat * (1.0 + ld(scale, in_f32, mrow * D + d))
                               + ld(shift, in_f32, mrow * D + d);
            }
            mean[n] = mu;
            rstd[n] = r;
        }
    }
    return 0;
}

/*
 * Backward.  dy, x [T,D]; scale as in the forward; dx [T,D];
 * dshift, dscale [nseg,D] (per segment) or [T,D] (per token), all double.
 * Returns 0, 1 for bad arguments, 2 if scratch memory could not be obtained.
 */
int lnmod_oracle_backward(const void *dy, const void *x, const void *scale, int in_f32,
                          const int64_t *cu, int64_t nseg, int64_t D, double eps, int mod,
                          double *dx, double *dshift, double *dscale)
{
    if (!cu || nseg < 0 || D <= 0) return 1;
    if (mod != LNMOD_ORACLE_PER_SEGMENT && mod != LNMOD_ORACLE_PER_TOKEN) return 1;
    for (int64_t m = 0; m < nseg; ++m)
        if (cu[m] < 0 || cu[m + 1] < cu[m]) return 1;
    const int64_t T = nseg > 0 ? cu[nseg] : 0;

    /* the statistics of every row, recomputed here from x */
    double *mu = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
    double *r = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
    if (!mu || !r) { free(mu); free(r); return 2; }

    for (int64_t m = 0; m < nseg; ++m) {
        const int64_t n0 = cu[m], n1 = cu[m + 1];
#pragma omp parallel for schedule(static)
        for (int64_t n = n0; n < n1; ++n) {
            row_stats(x, in_f32, n, D, eps, &mu[n], &r[n]);
            const int64_t mrow = (mod == LNMOD_ORACLE_PER_TOKEN) ? n : m;
            double s1 = 0.0, s2 = 0.0;
            for (int64_t d = 0; d < D; ++d) {
                double g = ld(dy, in_f32, n * D + d) * (1.0 + ld(scale, in_f32, mrow * D + d));
                double xhat = (ld(x, in_f32, n * D + d) - mu[n]) * r[n];
                s1 += g;
                s2 += g * xhat;
            }
            const double c1 = s1 / (double)D, c2 = s2 / (double)D;
            for (int64_t d = 0; d < D; ++d) {
                double g = ld(dy, in_f32, n * D + d) * (1.0 + ld(scale, in_f32, mrow * D + d));
                double xhat = (ld(x, in_f32, n * D + d) - mu[n]) * r[n];
                dx[n * D + d] = r[n] * (g - c1 - xhat * c2);
                if (mod == LNMOD_ORACLE_PER_TOKEN) {
                    dshift[n * D + d] = ld(dy, in_f32, n * D + d);
                    dscale[n * D + d] = ld(dy, in_f32, n * D + d) * xhat;
                }
            }
        }
    }

    if (mod == LNMOD_ORACLE_PER_SEGMENT) {
        /* token sums: for every (segment, feature) the tokens are added in index order.
           Threads own disjoint feature ranges [d0,d1); each walks the tokens top to bottom. */
        const int64_t FB = 64;
        for (int64_t m = 0; m < nseg; ++m) {
            const int64_t n0 = cu[m], n1 = cu[m + 1];
#pragma omp parallel for schedule(static)
            for (int64_t d0 = 0; d0 < D; d0 += FB) {
                const int64_t d1 = d0 + FB < D ? d0 + FB : D;
                for (int64_t d = d0; d < d1; ++d) {
                    dshift[m * D + d] = 0.0;
                    dscale[m * D + d] = 0.0;
                }
                for (int64_t n = n0; n < n1; ++n) {
                    for (int64_t d = d0; d < d1; ++d) {
                        double t = ld(dy, in_f32, n * D + d);
                        double xhat = (ld(x, in_f32, n * D + d) - mu[n]) * r[n];
                        dshift[m * D + d] += t;
                        dscale[m * D + d] += t * xhat;
                    }
                }
            }
        }
    }
    free(mu);
    free(r);
    return 0;
}
