"""torch.autograd wrappers over the C ABI: the three fused operators as differentiable functions.

Everything numerical runs in the HIP kernels; this module only allocates outputs with torch,
keeps what the backward needs and casts the float32 parameter gradients to the parameters' dtype.
Inputs must be contiguous CUDA tensors in bfloat16 or float32; work is enqueued on torch's
current stream.  Without the built library every call raises (there is no fallback).

    y        = ln_modulate(x, shift, scale)                      x [B,S,D]; shift, scale [B,D] or [B,S,D]
    y        = ln_modulate(x, shift, scale, cu_seqlens=cu)       x [T,D] packed; shift, scale [nseg,D]
    h, y     = gated_ln_modulate(x, u, gate, shift, scale)       h = x + gate*u, y = LN(h)(1+scale)+shift
    qn, kn   = qk_norm(q, k, wq, wk)                             RMS norm with weight of q and of k
"""
import torch

from . import lnmod


def _contig(*ts):
    for t in ts:
        if t is not None and not t.is_contiguous():
            raise ValueError("tensors must be contiguous")


class _LnModulate(torch.autograd.Function):
    """Sec. 3.3: forward saves x, scale and (optionally) the per-token statistics."""

    @staticmethod
    def forward(ctx, x, shift, scale, cu_seqlens, eps, save_stats):
        _contig(x, shift, scale, cu_seqlens)
        if cu_seqlens is None:
            y, mean, rstd = lnmod.forward(x, shift, scale, eps)
        else:
            y, mean, rstd = lnmod.forward_varlen(x, shift, scale, cu_seqlens, eps)
        ctx.eps = eps
        ctx.has_cu = cu_seqlens is not None
        ctx.param_dtype = shift.dtype
        if save_stats:
            ctx.save_for_backward(x, scale, cu_seqlens, mean, rstd)
        else:                                   # the backward forms them again from x
            ctx.save_for_backward(x, scale, cu_seqlens, None, None)
        return y

    @staticmethod
    def backward(ctx, dy):
        x, scale, cu, mean, rstd = ctx.saved_tensors
        dy = dy.contiguous()
        if ctx.has_cu:
            dx, dshift, dscale = lnmod.backward_varlen(dy, x, scale, cu, mean, rstd, ctx.eps)
        else:
            dx, dshift, dscale = lnmod.backward(dy, x, scale, mean, rstd, ctx.eps)
        return dx, dshift.to(ctx.param_dtype), dscale.to(ctx.param_dtype), None, None, None


def ln_modulate(x, shift, scale, eps=1e-6, cu_seqlens=None, save_stats=True):
    """y = LayerNorm(x) * (1 + scale) + shift (no affine, fp32 statistics).  save_stats=False keeps
    only x between the passes; the backward then recomputes mean and rstd."""
    return _LnModulate.apply(x, shift, scale, cu_seqlens, float(eps), bool(save_stats))


class _GatedLnModulate(torch.autograd.Function):
    """Sec. 4.4 "Gate + Norm": the residual update and the LayerNorm-Modulate after it."""

    @staticmethod
    def forward(ctx, x, u, gate, shift, scale, cu_seqlens, eps):
        _contig(x, u, gate, shift, scale, cu_seqlens)
        h, y, mean, rstd = lnmod.gated_forward(x, u, gate, shift, scale, cu_seqlens, eps)
        ctx.eps = eps
        ctx.param_dtype = gate.dtype
        ctx.save_for_backward(h, u, gate, scale, cu_seqlens, mean, rstd)
        return h, y

    @staticmethod
    def backward(ctx, dh, dy):
        h, u, gate, scale, cu, mean, rstd = ctx.saved_tensors
        dx, du, dgate, dshift, dscale = lnmod.gated_backward(dy.contiguous(), dh.contiguous(), h, u, gate,
                                                             scale, mean, rstd, cu, ctx.eps)
        pd = ctx.param_dtype
        return dx, du, dgate.to(pd), dshift.to(pd), dscale.to(pd), None, None


def gated_ln_modulate(x, u, gate, shift, scale, eps=1e-6, cu_seqlens=None):
    """h = x + gate * u (returned, it is the new residual stream) and y = LN(h) * (1 + scale) + shift."""
    return _GatedLnModulate.apply(x, u, gate, shift, scale, cu_seqlens, float(eps))


class _QkNorm(torch.autograd.Function):
    """Sec. 4.4 fused Q-Norm + K-Norm."""

    @staticmethod
    def forward(ctx, q, k, wq, wk, eps):
        _contig(q, k, wq, wk)
        qn, kn, rq, rk = lnmod.qknorm_forward(q, k, wq, wk, eps)
        ctx.eps = eps
        ctx.param_dtype = wq.dtype
        ctx.save_for_backward(q, k, wq, wk, rq, rk)
        return qn, kn

    @staticmethod
    def backward(ctx, dqn, dkn):
        q, k, wq, wk, rq, rk = ctx.saved_tensors
        dq, dk, dwq, dwk = lnmod.qknorm_backward(dqn.contiguous(), dkn.contiguous(), q, k, wq, wk, rq, rk,
                                                 ctx.eps)
        return dq, dk, dwq.to(ctx.param_dtype), dwk.to(ctx.param_dtype), None


def qk_norm(q, k, wq, wk, eps=1e-6):
    """q * rsqrt(mean(q^2) + eps) * wq and the same for k, in one launch."""
    return _QkNorm.apply(q, k, wq, wk, float(eps))
