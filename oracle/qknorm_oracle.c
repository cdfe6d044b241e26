/*
 * qknorm_oracle.c -- float64 CPU oracle for the fused Q-Norm + K-Norm operator.
 *
 * TEST INFRASTRUCTURE ONLY.  Slow, plain definition that the GPU path is checked against.  It
 * shares no code, header, table or helper with the HIP library (nor with the other oracle files)
 * and is never called from the product path; only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may load it.
 *
 * The paper lists "Q-Norm + K-Norm" among its fused operator chains (Sec. 4.4) and says nothing
 * more about it.  The definition used here is the query/key normalisation of MMDiT-style
 * attention blocks: a root-mean-square normalisation with a learned per-feature weight, applied
 * to the query rows and to the key rows before attention.  For one of the two tensors, x [N,D]
 * with weight w [D]:
 *
 *   ms_n   = (1/D) sum_d x[n,d]^2
 *   r_n    = 1 / sqrt(ms_n + eps)
 *   xhat   = x[n,d] * r_n
 *   y[n,d] = xhat * w[d]                      r_n is saved for the backward
 *
 *   g[n,d]  = dy[n,d] * w[d]
 *   c_n     = (1/D) sum_d g[n,d] * xhat[n,d]
 *   dx[n,d] = r_n * (g[n,d] - xhat[n,d] * c_n)
 *   dw[d]   = sum_n dy[n,d] * xhat[n,d]       over every row, in index order
 *
 * The operator is this, once for (q, wq) and once for (k, wk); the two halves do not interact,
 * so the functions below take one tensor and the caller invokes them for each.  The row length D
 * is whatever the caller normalises over: the whole projection width, or one head when the
 * tensor is viewed as [N*heads, head_dim].  The backward recomputes r from x.
 * Inputs arrive as double or as float (in_f32 != 0: an exact carrier of bf16/fp32 values);
 * every operation is done in double.  OpenMP only distributes independent rows / features.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

static inline double ld(const void *p, int in_f32, int64_t i)
{
    return in_f32 ? (double)((const float *)p)[i] : ((const double *)p)[i];
}

/* Forward of one tensor.  x [N,D], w [D]; y [N,D], rstd [N] in double.  Returns 0, or 1. */
int qknorm_oracle_forward(const void *x, const void *w, int in_f32, int64_t N, int64_t D,
                          double eps, double *y, double *rstd)
{
    if (N < 0 || D <= 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double s = 0.0;
        for (int64_t d = 0; d < D; ++d) {
            const double v = ld(x, in_f32, n * D + d);
            s += v * v;
        }
        const double r = 1.0 / sqrt(s / (double)D + eps);
        for (int64_t d = 0; d < D; ++d)
            y[n * D + d] = (ld(x, in_f32, n * D + d) * r) * ld(w, in_f32, d);
        rstd[n] = r;
    }
    return 0;
}

/*
 * Backward of one tensor.  dy, x [N,D], w [D]; dx [N,D], dw [D] in double.
 * Returns 0, 1 for bad arguments, 2 if scratch memory could not be obtained.
 */
int qknorm_oracle_backward(const void *dy, const void *x, const void *w, int in_f32, int64_t N,
                           int64_t D, double eps, double *dx, double *dw)
{
    if (N < 0 || D <= 0) return 1;
    double *r = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
    if (!r) return 2;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double s = 0.0;
        for (int64_t d = 0; d < D; ++d) {
            const double v = ld(x, in_f32, n * D + d);
            s += v * v;
        }
        r[n] = 1.0 / sqrt(s / (double)D + eps);
        double sc = 0.0;
        for (int64_t d = 0; d < D; ++d) {
            const double g = ld(dy, in_f32, n * D + d) * ld(w, in_f32, d);
            const double xhat = ld(x, in_f32, n * D + d) * r[n];
            sc += g * xhat;
        }
        const double c = sc / (double)D;
        for (int64_t d = 0; d < D; ++d) {
            const double g = ld(dy, in_f32, n * D + d) * ld(w, in_f32, d);
            const double xhat = ld(x, in_f32, n * D + d) * r[n];
            dx[n * D + d] = r[n] * (g - xhat * c);
        }
    }
    /* weight gradient: every row, in index order; threads own disjoint feature ranges */
    const int64_t FB = 64;
#pragma omp parallel for schedule(static)
    for (int64_t d0 = 0; d0 < D; d0 += FB) {
        const int64_t d1 = d0 + FB < D ? d0 + FB : D;
        for (int64_t d = d0; d < d1; ++d) dw[d] = 0.0;
        for (int64_t n = 0; n < N; ++n)
            for (int64_t d = d0; d < d1; ++d)
                dw[d] += ld(dy, in_f32, n * D + d) * (ld(x, in_f32, n * D + d) * r[n]);
    }
    free(r);
    return 0;
}
