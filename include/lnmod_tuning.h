/*
 * lnmod_tuning.h -- tuning interface of the fused LayerNorm-Modulate library (not part of the
 * operator API in lnmod.h; no caller of the operators needs it).
 *
 * Every kernel family picks its launch shape from a table that was measured on MI355X, one entry
 * per 512 features of row width.  This call replaces that choice for one family, process-wide,
 * so that a sweep can time the candidates of an entry through the same entry points the tables
 * serve (`python -m paper_2605_17923_amd.tune`).  Results do not depend on the shape beyond the
 * order of fp32 summation.
 *
 *   K        waves that share one row                         1..16
 *   VPL      16-byte chunks of the row each lane holds         1..6
 *   R        rows a block works on per step                    1..2
 *   per_cu   resident blocks per compute unit that the grid is sized for   1..16
 *
 * A launch whose row does not fit K * VPL * 64 chunks, or whose (K, VPL) was not compiled for the
 * family and element type, fails with LNMOD_ELAUNCH and enqueues nothing; it never computes on
 * part of a row.  K == 0 removes the override.  The setting is a plain global: change it only
 * while no other thread is inside a library call.  A backward family's workspace size follows its
 * shape: call the *_workspace_bytes query again after changing it.
 */
#ifndef LNMOD_TUNING_H
#define LNMOD_TUNING_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LNMOD_TUNE_FORWARD = 0,             /* lnmod_forward / _varlen, LNMOD_PER_SAMPLE              */
    LNMOD_TUNE_BACKWARD = 1,            /* lnmod_backward / _varlen with saved statistics          */
    LNMOD_TUNE_BACKWARD_RECOMPUTE = 2,  /* the same without saved statistics                       */
    LNMOD_TUNE_TOKEN_FORWARD = 3,       /* LNMOD_PER_TOKEN forward                                 */
    LNMOD_TUNE_TOKEN_BACKWARD = 4,      /* LNMOD_PER_TOKEN backward                                */
    LNMOD_TUNE_GATED_FORWARD = 5,       /* lnmod_gated_forward                                     */
    LNMOD_TUNE_GATED_BACKWARD = 6,      /* lnmod_gated_backward                                    */
    LNMOD_TUNE_QKNORM_FORWARD = 7,      /* lnmod_qknorm_forward, rows wider than one head (more    */
    LNMOD_TUNE_QKNORM_BACKWARD = 8      /* than 32 chunks); R must be 2.  lnmod_qknorm_backward    */
} lnmod_tune_family;

/* Returns LNMOD_OK, or LNMOD_EINVAL for an unknown family or a value outside the ranges above. */
int lnmod_tuning_set_shape(int family, int K, int VPL, int R, int per_cu);

/* The shape the family's table gives for rows of D elements of `dtype` (LNMOD_BF16 / LNMOD_F32),
 * ignoring any override; out receives K, VPL, R, per_cu (host pointer to 4 ints).
 * LNMOD_EINVAL for an unknown family or dtype or NULL out, LNMOD_EUNSUPPORTED for D. */
int lnmod_tuning_table_shape(int family, int64_t D, int dtype, int* out);

#ifdef __cplusplus
}
#endif
#endif
