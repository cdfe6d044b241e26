/*
 * lnmod_sched.h -- host-side C ABI of the dual-constraint bucket sizing and its cost-model fit
 * (paper Sec. 3.2).  No device is touched; every pointer is a HOST pointer; nothing is allocated
 * beyond the call's own stack; the functions are reentrant.
 *
 * A bucket is a data shape with logical sequence length S (text plus visual tokens).  Its batch
 * size is the smaller of a memory bound, linear in S, and a compute bound, polynomial in S with
 * the fitted exponent p of the attention cost, and never below one (Eq. 2):
 *
 *     B_shape = max(1, min(floor(M_mem / S), floor(M_comp / S^p)))
 *
 * p and M_comp come from measured step times of (B, S) pairs: the model
 * step_time ~ a + b * B * S^p is fitted by ordinary least squares for every p on a grid over
 * [p_lo, p_hi] (the paper searches [1.6, 2.4]; the grid step is not stated and is an argument
 * here), the p with the largest coefficient of determination R^2 is kept, and
 * M_comp = (target_sync - a) / b for a chosen target step time.
 */
#ifndef LNMOD_SCHED_H
#define LNMOD_SCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Eq. 2.  S >= 1; M_mem, M_comp finite and >= 0; p finite.  All arithmetic in double; S^p by
 * the C library's pow().  Returns B_shape >= 1, or 0 for invalid arguments.
 */
int64_t lnmod_bucket_batch_size(int64_t S, double M_mem, double M_comp, double p);

/* Eq. 2 for n buckets: out[i] = lnmod_bucket_batch_size(S[i], ...).  Returns 0, or 1 for invalid
 * arguments (NULL pointer with n > 0, n < 0). */
int lnmod_bucket_batch_sizes(const int64_t* S, int64_t n, double M_mem, double M_comp, double p,
                             int64_t* out);

/*
 * Cost-model fit (Sec. 3.2).  B, S, step_time: n measurements.  The grid is p_lo, p_lo + p_step,
 * ... up to and including p_hi (within 1e-9); for each p the least-squares line of step_time on
 * z = B * S^p gives (a, b) and R^2 = 1 - SSE/SST; the first grid point with the largest R^2 wins.
 * Outputs: *a, *b, *p, *r2.  Returns 0; 1 for invalid arguments (NULL pointer, n < 2,
 * p_step <= 0, p_hi < p_lo, non-finite input, B or S < 1); 2 if the fit is degenerate at every
 * grid point (all z equal, or all step times equal).
 */
int lnmod_fit_cost_model(const int64_t* B, const int64_t* S, const double* step_time, int64_t n,
                         double p_lo, double p_hi, double p_step,
                         double* a, double* b, double* p, double* r2);

/* M_comp = (target_sync - a) / b (Sec. 3.2).  Returns 0 when b <= 0 or the result is not a
 * positive finite number (no compute bound can be derived). */
double lnmod_comp_bound(double target_sync, double a, double b);

#ifdef __cplusplus
}
#endif
#endif /* LNMOD_SCHED_H */
