/*
 * gated_oracle.c -- float64 CPU oracle for the gated-residual + LayerNorm-Modulate operator.
 *
 * TEST INFRASTRUCTURE ONLY.  Slow, plain definition that the GPU path is checked against.  It
 * shares no code, header, table or helper with the HIP library (nor with the other oracle
 * file: the few lines both need are written out in each) and is never called from the product
 * path; only the tests, the smoke check and the benchmark's cpu_baseline leg may load it.
 *
 * The paper lists "Gate + Norm" among its fused operator chains (Sec. 4.4) without defining
 * it.  The definition used here is the one a DiT block with adaptive LayerNorm gives: the
 * branch output u, scaled by the timestep-conditioned gate, is added to the residual stream,
 * and the sum goes straight into the next LayerNorm-Modulate (Sec. 3.3 for that part):
 *
 *   t[n,d]  = x[n,d] + gate[m,d] * u[n,d]
 *   h[n,d]  = Q(t[n,d])                                the residual stream as it is stored
 *   mu_n    = (1/D) sum_d h[n,d]
 *   var_n   = (1/D) sum_d (h[n,d] - mu_n)^2            two passes, biased
 *   r_n     = 1 / sqrt(var_n + eps)
 *   hhat    = (h[n,d] - mu_n) * r_n
 *   y[n,d]  = hhat * (1 + scale[m,d]) + shift[m,d]
 *
 * Q is the rounding to the storage type of h, because the next operator and the backward pass
 * read h from memory: Q = identity (quant 0, used by the differentiation pins), round to
 * nearest even to float32 (quant 1), or that followed by round to nearest even to bfloat16
 * (quant 2: what a float32 fused multiply-add followed by one bf16 store produces).
 *
 * Backward, given dy (gradient of y) and dh (gradient that reaches h along the residual
 * stream), with Q treated as the identity:
 *
 *   g       = dy[n,d] * (1 + scale[m,d])
 *   c1_n    = (1/D) sum_d g ;  c2_n = (1/D) sum_d g * hhat
 *   dx[n,d] = dh[n,d] + r_n * (g - c1_n - hhat * c2_n)        gradient of x (and of t)
 *   du[n,d] = gate[m,d] * dx[n,d]
 *   dgate[m,d]  = sum_{n in m} u[n,d] * dx[n,d]
 *   dshift[m,d] = sum_{n in m} dy[n,d]
 *   dscale[m,d] = sum_{n in m} dy[n,d] * hhat[n,d]
 *
 * m is the segment that contains token n (a sample of a fixed-length batch is a segment of
 * length S).  The backward recomputes mu and r from h.  Sums over tokens run in index order.
 * Inputs arrive as double or as float (in_f32 != 0: an exact carrier of bf16/fp32 values);
 * every operation is done in double.  OpenMP only distributes independent rows / features.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline double ld(const void *p, int in_f32, int64_t i)
{
    return in_f32 ? (double)((const float *)p)[i] : ((const double *)p)[i];
}

/* float32 -> nearest bfloat16 (ties to even), returned as a float32 value */
static float to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return f;            /* NaN stays NaN */
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return f;
}

static double quantise(double t, int quant)
{
    if (quant == 0) return t;
    float f = (float)t;                                        /* round to nearest even */
    if (quant == 2) f = to_bf16(f);
    return (double)f;
}

static int check_table(const int64_t *cu, int64_t nseg)
{
    for (int64_t m = 0; m < nseg; ++m)
        if (cu[m] < 0 || cu[m + 1] < cu[m]) return 1;
    return 0;
}

/* mean and reciprocal standard deviation of one row of doubles (two passes) */
static void row_stats(const double *h, int64_t D, double eps, double *mu_out, double *r_out)
{
    double s = 0.0;
    for (int64_t d = 0; d < D; ++d) s += h[d];
    const double mu = s / (double)D;
    double q = 0.0;
    for (int64_t d = 0; d < D; ++d) q += (h[d] - mu) * (h[d] - mu);
    *mu_out = mu;
    *r_out = 1.0 / sqrt(q / (double)D + eps);
}

/*
 * Forward.  x, u [T,D]; gate, shift, scale [nseg,D]; cu [nseg+1] token offsets.
 * h, y [T,D], mean, rstd [T] in double.  Returns 0, or 1 for bad arguments.
 */
int gated_oracle_forward(const void *x, const void *u, const void *gate, const void *shift,
                         const void *scale, int in_f32, const int64_t *cu, int64_t nseg,
                         int64_t D, double eps, int quant,
                         double *h, double *y, double *mean, double *rstd)
{
    if (!cu || nseg < 0 || D <= 0 || quant < 0 || quant > 2) return 1;
    if (check_table(cu, nseg)) return 1;
    for (int64_t m = 0; m < nseg; ++m) {
        const int64_t n0 = cu[m], n1 = cu[m + 1];
#pragma omp parallel for schedule(static)
        for (int64_t n = n0; n < n1; ++n) {
            for (int64_t d = 0; d < D; ++d) {
                const double t = ld(x, in_f32, n * D + d)
                                 + ld(gate, in_f32, m * D + d) * ld(u, in_f32, n * D + d);
                h[n * D + d] = quantise(t, quant);
            }
            double mu, r;
            row_stats(h + n * D, D, eps, &mu, &r);
            for (int64_t d = 0; d < D; ++d) {
                const double hhat = (h[n * D + d] - mu) * r;
                y[n * D + d] = hhat * (1.0 + ld(scale, in_f32, m * D + d))
                               + ld(shift, in_f32, m * D + d);
            }
            mean[n] = mu;
            rstd[n] = r;
        }
    }
    return 0;
}

/*
 * Backward.  dy, dh, h, u [T,D]; gate, scale [nseg,D]; dx, du [T,D];
 * dgate, dshift, dscale [nseg,D], all outputs double.
 * Returns 0, 1 for bad arguments, 2 if scratch memory could not be obtained.
 */
int gated_oracle_backward(const void *dy, const void *dh, const void *h, const void *u,
                          const void *gate, const void *scale, int in_f32, const int64_t *cu,
                          int64_t nseg, int64_t D, double eps,
                          double *dx, double *du, double *dgate, double *dshift, double *dscale)
{
    if (!cu || nseg < 0 || D <= 0) return 1;
    if (check_table(cu, nseg)) return 1;
    const int64_t T = nseg > 0 ? cu[nseg] : 0;
    double *mu = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
    double *r = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
    if (!mu || !r) { free(mu); free(r); return 2; }

    for (int64_t m = 0; m < nseg; ++m) {
        const int64_t n0 = cu[m], n1 = cu[m + 1];
#pragma omp parallel for schedule(static)
        for (int64_t n = n0; n < n1; ++n) {
            /* statistics of the stored row */
            double s = 0.0;
            for (int64_t d = 0; d < D; ++d) s += ld(h, in_f32, n * D + d);
            mu[n] = s / (double)D;
            double q = 0.0;
            for (int64_t d = 0; d < D; ++d) {
                const double c = ld(h, in_f32, n * D + d) - mu[n];
                q += c * c;
            }
            r[n] = 1.0 / sqrt(q / (double)D + eps);

            double s1 = 0.0, s2 = 0.0;
            for (int64_t d = 0; d < D; ++d) {
                const double g = ld(dy, in_f32, n * D + d) * (1.0 + ld(scale, in_f32, m * D + d));
                const double hhat = (ld(h, in_f32, n * D + d) - mu[n]) * r[n];
                s1 += g;
                s2 += g * hhat;
            }
            const double c1 = s1 / (double)D, c2 = s2 / (double)D;
            for (int64_t d = 0; d < D; ++d) {
                const double g = ld(dy, in_f32, n * D + d) * (1.0 + ld(scale, in_f32, m * D + d));
                const double hhat = (ld(h, in_f32, n * D + d) - mu[n]) * r[n];
                const double dln = r[n] * (g - c1 - hhat * c2);
                dx[n * D + d] = ld(dh, in_f32, n * D + d) + dln;
                du[n * D + d] = ld(gate, in_f32, m * D + d) * dx[n * D + d];
            }
        }
    }

    /* token sums in index order; threads own disjoint feature ranges */
    const int64_t FB = 64;
    for (int64_t m = 0; m < nseg; ++m) {
        const int64_t n0 = cu[m], n1 = cu[m + 1];
#pragma omp parallel for schedule(static)
        for (int64_t d0 = 0; d0 < D; d0 += FB) {
            const int64_t d1 = d0 + FB < D ? d0 + FB : D;
            for (int64_t d = d0; d < d1; ++d) {
                dgate[m * D + d] = 0.0;
                dshift[m * D + d] = 0.0;
                dscale[m * D + d] = 0.0;
            }
            for (int64_t n = n0; n < n1; ++n) {
                for (int64_t d = d0; d < d1; ++d) {
                    const double t = ld(dy, in_f32, n * D + d);
                    const double hhat = (ld(h, in_f32, n * D + d) - mu[n]) * r[n];
                    dgate[m * D + d] += ld(u, in_f32, n * D + d) * dx[n * D + d];
                    dshift[m * D + d] += t;
                    dscale[m * D + d] += t * hhat;
                }
            }
        }
    }
    free(mu);
    free(r);
    return 0;
}
