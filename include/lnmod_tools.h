/*
 * lnmod_tools.h -- C ABI of liblnmod_tools.so, the measurement companion of the fused
 * LayerNorm-Modulate library.  Nothing here is part of the operator interface (include/lnmod.h) and
 * no caller of the operators needs it: the benchmark and the launch-shape sweep do.  It is built
 * from the same kernel sources as liblnmod.so and holds
 *   - bandwidth references: a plain copy and stream probes of given read/write mixtures,
 *   - the comparators of the fused-against-unfused measurement (Sec. 3.3, 3.4 of the paper argue
 *     against the decoupled chain; Sec. 4.4 compares with it),
 *   - "shaped" forms of lnmod_forward / lnmod_backward that take the launch shape as an argument
 *     of the call instead of looking it up in the measured tables, so that candidates can be timed
 *     through the same code without any process-wide setting,
 *   - queries that report the measured tables and name the kernels a call launches.
 * Conventions (device pointers, caller's stream, no allocation, no synchronisation, status codes,
 * validation before any HIP call) are those of lnmod.h.
 */
#ifndef LNMOD_TOOLS_H
#define LNMOD_TOOLS_H

#include <stddef.h>
#include <stdint.h>

#include "lnmod.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * lnmod_copy: plain 16-byte-vector device copy of `bytes` bytes (a multiple of 16), the practical
 * bandwidth ceiling the kernels are compared with.
 */
int lnmod_copy(const void* src, void* dst, size_t bytes, void* stream);

/*
 * lnmod_stream_probe: the copy's access pattern with a chosen number of read and write streams, to
 * show what the memory system gives to reads, to writes and to the mixtures the kernels produce.
 * in[i] (i < reads) and out[j] (j < writes) are host arrays of device pointers to buffers of `bytes`
 * bytes each (a multiple of 16; a tail shorter than one piece of 4 or 8 KB is left out).  Every
 * output is the 32-bit-lane sum of the inputs plus j (a position-dependent pattern when reads is 0).
 * With writes == 0 the inputs are read and summed, and out[0] must point to 1 KB that is normally
 * not written.  Supported (reads, writes): (1,0) (0,1) (1,1) (2,1) (2,2) (3,1) (3,3) (4,2).
 * blocks, waves (per block, 1..8) and vecs (16-byte vectors per lane and step: 1, 2, 4 or 8) give
 * the launch; all three 0 selects the mixture's default (the best of a sweep).
 * LNMOD_EINVAL for any other mixture or launch, a NULL pointer or bytes not a multiple of 16.
 */
int lnmod_stream_probe(const void* const* in, int reads, void* const* out, int writes, size_t bytes,
                       int blocks, int waves, int vecs, void* stream);

/*
 * lnmod_unfused_forward: the decoupled chain: kernel 1 writes xhat (I/O dtype) and the statistics
 * to HBM, kernel 2 reads xhat back and applies the per-sample modulation.  xhat_tmp: [B*S, D]
 * scratch in the I/O dtype.
 */
int lnmod_unfused_forward(const void* x, const void* shift, const void* scale,
                          int64_t B, int64_t S, int64_t D, float eps, void* stream,
                          void* xhat_tmp, void* y, float* mean, float* rstd, int dtype);

/*
 * lnmod_gate_residual: only h = x + gate*u (per-sample gate [B, D]), the first kernel of the unfused
 * chain "residual update, then lnmod_forward on h" that lnmod_gated_forward is compared with.
 */
int lnmod_gate_residual(const void* x, const void* u, const void* gate, int64_t B, int64_t S,
                        int64_t D, void* stream, void* h, int dtype);

/*
 * Launch shape of a row kernel:
 *   shape[0] K        waves that share one row                         1..16
 *   shape[1] VPL      16-byte chunks of the row each lane holds         1..6
 *   shape[2] R        rows a block works on per step                    1..2
 *   shape[3] per_cu   resident blocks per compute unit that the grid is sized for   1..16
 *   shape[4] clusters 0: the plan's choice; 1..256: that many groups of blocks, each streaming
 *                     through its own contiguous share of the rows (per-sample kernels only)
 *   shape[5] interleave  0: consecutive blocks form a cluster (every cluster is spread over all
 *                     XCDs); 1: cluster = block index modulo the cluster count, so that with 8
 *                     clusters each cluster's blocks all sit on one XCD
 *   shape[6] flat     per-sample forward only: 1 runs one loop over all rows of a block's region and
 *                     reloads the modulation registers where the segment changes, 2 runs one loop per
 *                     segment, 0 leaves the choice to the launcher
 * (a host array of 7 ints).
 * Results do not depend on the shape beyond the order of fp32 summation.  A shape whose K * VPL *
 * 64 chunks do not cover the row, or whose (K, VPL) is not compiled for the kernel family and
 * element type, fails with LNMOD_ELAUNCH and enqueues nothing; values outside the ranges above are
 * LNMOD_EINVAL.  shape == NULL means the measured table's entry, i.e. what lnmod.h's calls use.
 */

typedef enum {
    LNMOD_FAMILY_FORWARD = 0,             /* lnmod_forward / _varlen, LNMOD_PER_SAMPLE              */
    LNMOD_FAMILY_BACKWARD = 1,            /* lnmod_backward / _varlen with saved statistics          */
    LNMOD_FAMILY_BACKWARD_RECOMPUTE = 2,  /* the same without saved statistics                       */
    LNMOD_FAMILY_TOKEN_FORWARD = 3,       /* LNMOD_PER_TOKEN forward                                 */
    LNMOD_FAMILY_TOKEN_BACKWARD = 4,      /* LNMOD_PER_TOKEN backward                                */
    LNMOD_FAMILY_GATED_FORWARD = 5,       /* lnmod_gated_forward                                     */
    LNMOD_FAMILY_GATED_BACKWARD = 6,      /* lnmod_gated_backward                                    */
    LNMOD_FAMILY_QKNORM_FORWARD = 7,      /* lnmod_qknorm_forward, rows wider than one head          */
    LNMOD_FAMILY_QKNORM_BACKWARD = 8      /* lnmod_qknorm_backward, rows wider than one head         */
} lnmod_family;

/* The shape a family's measured table gives for rows of D elements of `dtype` and (where the entry
 * depends on it; 0 = unknown) `tokens` rows; out: host pointer to 4 ints.  LNMOD_EINVAL for an
 * unknown family or dtype or NULL out, LNMOD_EUNSUPPORTED for D. */
int lnmod_table_shape(int family, int64_t D, int dtype, int64_t tokens, int* out);

/*
 * lnmod_forward / lnmod_forward_varlen with the launch shape given (cu_seqlens == NULL: B samples
 * of S tokens, B_or_nseg = B, S_or_T = S; else a packed batch, B_or_nseg = nseg, S_or_T = T and mod
 * must be LNMOD_PER_SAMPLE).  Everything else as in lnmod.h.
 */
int lnmod_forward_shaped(const int* shape, const void* x, const void* shift, const void* scale,
                         const int32_t* cu_seqlens, int64_t B_or_nseg, int64_t S_or_T, int64_t D,
                         float eps, void* stream, void* y, float* mean, float* rstd, int dtype,
                         int mod);

/*
 * lnmod_backward / lnmod_backward_varlen with the launch shape given.  The workspace size follows
 * the shape: lnmod_backward_workspace_bytes_shaped(shape, ...).
 */
int lnmod_backward_shaped(const int* shape, const void* dy, const void* x, const void* scale,
                          const int32_t* cu_seqlens, int64_t B_or_nseg, int64_t S_or_T, int64_t D,
                          float eps, void* stream, const float* mean, const float* rstd, void* dx,
                          void* dshift, void* dscale, void* workspace, size_t workspace_bytes,
                          int dtype, int mod);
size_t lnmod_backward_workspace_bytes_shaped(const int* shape, int64_t B_or_nseg,
                                             int64_t total_tokens, int64_t D, int mod);

/*
 * Writes into buf (host, n bytes, NUL-terminated, truncated if need be) the kernel instantiations
 * and grids that the forward (backward = 0) or backward call with these arguments launches, e.g.
 * "fwd_split_kernel<bf16_io, 2, 5, 2, true, 0, true> grid=256 block=320 clusters=1"; template
 * arguments in the order of the kernel's parameter list, as a profiler prints them.  `recompute`:
 * the backward is given no saved statistics.  A benchmark compares this text with the one recorded
 * beside a counter measurement to know whether the measurement still describes the launch.
 * Returns the length written (0 for invalid arguments).  Host-only, touches no device.
 */
int lnmod_describe_launch(int backward, const int* shape, int64_t B_or_nseg, int64_t S_or_T,
                          int varlen, int64_t D, int dtype, int mod, int recompute, char* buf,
                          size_t n);

#ifdef __cplusplus
}
#endif
#endif /* LNMOD_TOOLS_H */
