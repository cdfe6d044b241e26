/*
 * lnmod.h -- C ABI of the MI355X (gfx950) fused LayerNorm-Modulate (AdaLN) library.
 *
 * The operator is the one the paper fuses in Sec. 3.3 ("Fused LayerNorm-Modulate kernels"):
 * for every token row, mean and variance over the hidden dimension D, normalisation, and the
 * modulation by the timestep-conditioned shift/scale, in one launch; the statistics are kept in
 * global memory for the backward pass; the backward pass returns dx and the modulation
 * gradients reduced along the token axis with fp32 accumulation (Sec. 3.3, Sec. 4.5).
 * Written out (LayerNorm without affine, biased variance, eps inside the square root):
 *
 *     mean_n = (1/D) sum_d x[n,d]            rstd_n = 1/sqrt((1/D) sum_d (x[n,d]-mean_n)^2 + eps)
 *     xhat   = (x[n,d] - mean_n) * rstd_n    y[n,d] = xhat * (1 + scale[m,d]) + shift[m,d]
 *     g      = dy[n,d] * (1 + scale[m,d])    c1 = (1/D) sum_d g      c2 = (1/D) sum_d g*xhat
 *     dx[n,d] = rstd_n * (g - c1 - xhat*c2)
 *     dshift[m,d] = sum_{n in m} dy[n,d]     dscale[m,d] = sum_{n in m} dy[n,d]*xhat[n,d]
 *
 * m is the modulation row of token n: its sample (LNMOD_PER_SAMPLE), its packed segment
 * (the *_varlen calls) or the token itself (LNMOD_PER_TOKEN, no sum).
 *
 * Conventions common to every call
 *   - Every pointer is a DEVICE pointer (memory of the current HIP device) unless the comment
 *     says "host".  The caller owns every buffer.  The library allocates nothing, frees
 *     nothing and never synchronises: kernels are enqueued on `stream` (a hipStream_t passed
 *     as void*; NULL is the default stream) and the call returns at once.
 *   - Tensors are dense and row-major with D contiguous: x, y, dy, dx are [N, D], N tokens.
 *   - `dtype` is the element type of x, y, dy, dx, shift, scale (LNMOD_BF16 or LNMOD_F32).
 *     All arithmetic is fp32; bf16 results are rounded once, to nearest even, at the store.
 *     mean, rstd and the reduced dshift/dscale are always float32.
 *   - Supported D: a multiple of 8 (bf16) or 4 (fp32), 8 <= D <= 8192.  Every tensor pointer
 *     must be 16-byte aligned.
 *   - Inputs and outputs must not overlap.  Outputs are overwritten in full; nothing is
 *     accumulated into them.  Results are bitwise reproducible for equal inputs and shapes.
 *   - The return value is the only error channel (no exceptions, no abort, nothing printed).
 *     Arguments are validated before any HIP call, so a bad call enqueues nothing.
 *       LNMOD_EINVAL        NULL required pointer; negative size; eps not finite or <= 0;
 *                           unknown dtype or mod; token count at or above 2^31; more than
 *                           2^24 - 1 samples or segments
 *       LNMOD_EUNSUPPORTED  D outside the supported set
 *       LNMOD_EALIGN        a tensor pointer is not 16-byte aligned
 *       LNMOD_EWORKSPACE    workspace NULL or smaller than lnmod_backward_workspace_bytes()
 *       LNMOD_ELAUNCH       the HIP runtime reported an error for the launch
 *     N == 0 returns LNMOD_OK; per-sample dshift/dscale of B > 0 samples are then zero-filled.
 */
#ifndef LNMOD_H
#define LNMOD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LNMOD_OK = 0,
    LNMOD_EINVAL = 1,
    LNMOD_EUNSUPPORTED = 2,
    LNMOD_EALIGN = 3,
    LNMOD_EWORKSPACE = 4,
    LNMOD_ELAUNCH = 5
} lnmod_status;

typedef enum { LNMOD_BF16 = 0, LNMOD_F32 = 1 } lnmod_dtype;

typedef enum {
    LNMOD_PER_SAMPLE = 0, /* shift, scale: [B, D] */
    LNMOD_PER_TOKEN = 1   /* shift, scale: [B, S, D] */
} lnmod_mod;

/*
 * Forward (Sec. 3.3, forward kernel: statistics, normalisation and modulation in one launch,
 * statistics saved).  x, y: [B*S, D]; shift, scale: [B, D] or [B, S, D] by `mod`;
 * mean, rstd: float32 [B*S] (written).  mean and rstd may both be NULL (one alone is
 * LNMOD_EINVAL): the statistics are then not stored, for callers that need only y (inference,
 * or a backward that recomputes them, see lnmod_backward); y is the same bit for bit.
 */
int lnmod_forward(const void* x, const void* shift, const void* scale,
                  int64_t B, int64_t S, int64_t D, float eps, void* stream,
                  void* y, float* mean, float* rstd, int dtype, int mod);

/*
 * Backward (Sec. 3.3, backward: dx, and dshift/dscale by per-feature accumulation along the
 * sequence in fp32).  dy, x, dx: [B*S, D]; mean, rstd: what lnmod_forward saved for this x.
 * `shift` is not needed and may be NULL; `eps` is not needed (rstd is saved) and is only
 * validated.  mean and rstd may both be NULL (one alone is LNMOD_EINVAL): the statistics are
 * then formed again from x with `eps`, for callers that keep only x between the passes
 * (Sec. 3.3: nothing but the operator's output has to be stored); the result agrees with the
 * saved-statistics result to rounding.
 * LNMOD_PER_SAMPLE: dshift, dscale are float32 [B, D] and `workspace` must hold
 * lnmod_backward_workspace_bytes(B, B*S, D, mod) bytes (contents need no initialisation and
 * are garbage afterwards).  LNMOD_PER_TOKEN: dshift, dscale are [B, S, D] in the I/O dtype;
 * workspace may be NULL.
 */
int lnmod_backward(const void* dy, const void* x, const void* shift, const void* scale,
                   int64_t B, int64_t S, int64_t D, float eps, void* stream,
                   const float* mean, const float* rstd,
                   void* dx, void* dshift, void* dscale,
                   void* workspace, size_t workspace_bytes, int dtype, int mod);

/*
 * Forward on a packed batch of nseg segments of different lengths (the mixed image/video
 * batches of Sec. 3.2 laid end to end).  x, y: [T, D]; shift, scale: [nseg, D];
 * cu_seqlens: device int32 [nseg+1], non-decreasing, cu_seqlens[0] = 0, cu_seqlens[nseg] = T;
 * zero-length segments are allowed.  The table is read on the device only; a malformed table
 * gives unspecified values but no out-of-bounds access.  nseg plays B, T plays S.  mean and rstd
 * may both be NULL, as in lnmod_forward.
 */
int lnmod_forward_varlen(const void* x, const void* shift, const void* scale,
                         const int32_t* cu_seqlens, int64_t nseg, int64_t T, int64_t D,
                         float eps, void* stream,
                         void* y, float* mean, float* rstd, int dtype);

/*
 * Backward on a packed batch.  dshift, dscale: float32 [nseg, D]; the rows of zero-length
 * segments are written as zeros.  workspace: lnmod_backward_workspace_bytes(nseg, T, D,
 * LNMOD_PER_SAMPLE) bytes.  mean and rstd may both be NULL, as in lnmod_backward.
 */
int lnmod_backward_varlen(const void* dy, const void* x, const void* shift, const void* scale,
                          const int32_t* cu_seqlens, int64_t nseg, int64_t T, int64_t D,
                          float eps, void* stream,
                          const float* mean, const float* rstd,
                          void* dx, void* dshift, void* dscale,
                          void* workspace, size_t workspace_bytes, int dtype);

/*
 * lnmod_backward for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments and results as lnmod_backward (bit for bit: the same kernels and launch plan) without
 * `workspace` / `workspace_bytes`: the per-block partial sums go to a static device array of
 * LNMOD_STATIC_WORKSPACE_BYTES inside the library (one per GPU, held from the time the library's
 * code is loaded on that GPU until the process ends).  The call allocates nothing, frees nothing
 * and never synchronises.  A LNMOD_PER_SAMPLE problem whose partial sums need more than that
 * (about 1600 slots of 2*D floats at D = 5120) is refused with LNMOD_EWORKSPACE before anything is
 * enqueued; LNMOD_PER_TOKEN needs no workspace and is never refused for it.  Every call on a GPU
 * uses that GPU's one array: calls that may overlap in time on the same GPU (different streams,
 * different host threads) race on it and must be serialised by the caller; calls on one stream
 * are ordered and safe.  The array needs no clearing between calls (every slot that is read has
 * been written by the same call).
 */
#define LNMOD_STATIC_WORKSPACE_BYTES ((size_t)64 << 20)
int lnmod_backward_static(const void* dy, const void* x, const void* shift, const void* scale,
                          int64_t B, int64_t S, int64_t D, float eps, void* stream,
                          const float* mean, const float* rstd,
                          void* dx, void* dshift, void* dscale, int dtype, int mod);

/*
 * Bytes of device workspace the backward needs for its per-block partial sums of
 * dshift/dscale (Sec. 3.3: per-feature accumulation down the sequence; the partials of the
 * blocks are combined by a second, fixed-order kernel).  0 for LNMOD_PER_TOKEN and for invalid
 * arguments.  Host-only, touches no device.
 */
size_t lnmod_backward_workspace_bytes(int64_t B_or_nseg, int64_t total_tokens, int64_t D, int mod);

/* Static, NUL-terminated description of a status code (host pointer, never NULL). */
const char* lnmod_status_string(int status);

/*
 * Gated residual + LayerNorm-Modulate: the "Gate + Norm" chain the paper lists among its fused
 * operators (Sec. 4.4) without defining it; defined here as a DiT block with adaptive LayerNorm
 * has it around every LayerNorm-Modulate (Sec. 3.3):
 *
 *     h[n,d] = x[n,d] + gate[m,d]*u[n,d]     one fp32 fused multiply-add, rounded once (to nearest
 *                                            even) to the I/O dtype and stored: the residual stream
 *     y      = LayerNorm-Modulate of h as stored (formulas at the top), mean/rstd of h saved
 *
 * x, u, h, y: [N, D]; gate, shift, scale: [B, D] (cu_seqlens == NULL: B samples of S tokens;
 * B_or_nseg = B, S_or_T = S) or [nseg, D] (cu_seqlens a device int32 [nseg+1] table as in
 * lnmod_forward_varlen; B_or_nseg = nseg, S_or_T = T).  Errors as for lnmod_forward.
 */
int lnmod_gated_forward(const void* x, const void* u, const void* gate, const void* shift,
                        const void* scale, const int32_t* cu_seqlens, int64_t B_or_nseg,
                        int64_t S_or_T, int64_t D, float eps, void* stream,
                        void* h, void* y, float* mean, float* rstd, int dtype);

/*
 * Backward of the above.  dy: gradient of y; dh: gradient that reaches h along the residual
 * stream; h, mean, rstd: what lnmod_gated_forward produced; u, gate, scale: its inputs.
 *
 *     dx[n,d] = dh[n,d] + rstd_n*(g - c1 - hhat*c2)      (g, c1, c2 as at the top, with h for x)
 *     du[n,d] = gate[m,d]*dx[n,d]
 *     dgate[m,d] = sum_{n in m} u[n,d]*dx[n,d]    dshift, dscale as for lnmod_backward
 *
 * dx, du: [N, D] in the I/O dtype (dx is the gradient of x and of the incoming residual stream);
 * dgate, dshift, dscale: float32 [B, D] / [nseg, D], zeros for empty segments; the sums use the
 * fp32 dx before it is rounded.  workspace: lnmod_gated_backward_workspace_bytes() bytes, contents
 * need no initialisation.  `eps` is only validated.  Errors as for lnmod_backward.
 */
int lnmod_gated_backward(const void* dy, const void* dh, const void* h, const void* u,
                         const void* gate, const void* scale, const int32_t* cu_seqlens,
                         int64_t B_or_nseg, int64_t S_or_T, int64_t D, float eps, void* stream,
                         const float* mean, const float* rstd,
                         void* dx, void* du, float* dgate, float* dshift, float* dscale,
                         void* workspace, size_t workspace_bytes, int dtype);

/* Bytes of device workspace lnmod_gated_backward needs (0 for invalid arguments).  Host-only. */
size_t lnmod_gated_backward_workspace_bytes(int64_t B_or_nseg, int64_t total_tokens, int64_t D);

/*
 * Fused Q-Norm + K-Norm: the paper lists it among its fused operators (Sec. 4.4) without defining
 * it; defined here as the query/key normalisation of MMDiT-style attention blocks, a root-mean-
 * square normalisation with a learned weight, applied to both tensors by one launch:
 *
 *     rstd_n = 1/sqrt((1/D) sum_d x[n,d]^2 + eps)     y[n,d] = (x[n,d]*rstd_n) * w[d]
 *
 * for (x, w, y, rstd) = (q, wq, q_out, rstd_q) and (k, wk, k_out, rstd_k).  q, k, q_out, k_out:
 * [N, D] in the I/O dtype; wq, wk: [D] in the I/O dtype; rstd_q, rstd_k: float32 [N] (written).
 * N is the number of rows normalised (tokens, or tokens x heads when D is one head's width).
 * Errors as for lnmod_forward.
 */
int lnmod_qknorm_forward(const void* q, const void* k, const void* wq, const void* wk,
                         int64_t N, int64_t D, float eps, void* stream,
                         void* q_out, void* k_out, float* rstd_q, float* rstd_k, int dtype);

/*
 * Backward of the above, per tensor:  g = dy*w,  c_n = (1/D) sum_d g*xhat,
 * dx = rstd_n*(g - xhat*c_n),  dw[d] = sum_n dy[n,d]*xhat[n,d]  (xhat = x*rstd_n).
 * dq_out, dk_out: gradients of q_out, k_out; rstd_q, rstd_k: what the forward saved; dq, dk:
 * [N, D] in the I/O dtype; dwq, dwk: float32 [D], sums over all N rows in a fixed order (zeros
 * when N == 0).  workspace: lnmod_qknorm_backward_workspace_bytes(N, D) bytes, contents need no
 * initialisation.  `eps` is only validated.  Errors as for lnmod_backward.
 */
int lnmod_qknorm_backward(const void* dq_out, const void* dk_out, const void* q, const void* k,
                          const void* wq, const void* wk, int64_t N, int64_t D, float eps,
                          void* stream, const float* rstd_q, const float* rstd_k,
                          void* dq, void* dk, float* dwq, float* dwk,
                          void* workspace, size_t workspace_bytes, int dtype);

/* Bytes of device workspace lnmod_qknorm_backward needs (0 for invalid arguments).  Host-only. */
size_t lnmod_qknorm_backward_workspace_bytes(int64_t N, int64_t D);

#ifdef __cplusplus
}
#endif
#endif /* LNMOD_H */
