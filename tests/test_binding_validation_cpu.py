"""The convenience wrappers of the binding check every tensor before the C call (the C entry
points see addresses only, so a wrong shape, element type, layout or device would make the
kernels read out of bounds).  Shape, element type and layout are looked at before the device, so
all of these rejections can be exercised with host tensors; nothing here reaches the library."""
import pytest
import torch

from paper_2605_17923_amd import lnmod

B, S, D = 2, 6, 64
bf, f32 = torch.bfloat16, torch.float32


def t(*shape, dtype=bf):
    return torch.zeros(*shape, dtype=dtype)


def rejects(fn, *args, match=None, **kw):
    with pytest.raises(ValueError, match=match):
        fn(*args, **kw)


def test_forward_rejections():
    x, sh, sc = t(B, S, D), t(B, D), t(B, D)
    rejects(lnmod.forward, x, t(1, D).expand(B, D), sc, match="contiguous")        # stride-0 broadcast
    rejects(lnmod.forward, x, sh, t(B, D, dtype=f32), match="bfloat16")            # fp32 modulation, bf16 x
    rejects(lnmod.forward, t(B, S, D, dtype=f32), sh.float(), sc, match="float32")
    rejects(lnmod.forward, x, t(B + 1, D), t(B + 1, D), match="shape")
    rejects(lnmod.forward, x, t(B, D), t(B, S, D), match="shape")                  # shift per sample, scale per token
    rejects(lnmod.forward, x, t(D), t(D), match=r"\[B, D\]")
    rejects(lnmod.forward, t(B * S, D), sh, sc, match=r"\[B, S, D\]")
    rejects(lnmod.forward, t(B, S, 2 * D)[:, :, ::2], sh, sc, match="contiguous")  # strided x
    rejects(lnmod.forward, t(B, S, D, dtype=torch.float16), sh, sc, match="bfloat16 or float32")
    rejects(lnmod.forward, x, sh, sc, match="GPU")                                 # all consistent, but on the host


def test_backward_rejections():
    x, dy, sc = t(B, S, D), t(B, S, D), t(B, D)
    mean, rstd = t(B, S, dtype=f32), t(B, S, dtype=f32)
    rejects(lnmod.backward, t(B, S + 1, D), x, sc, mean, rstd, match="dy must have shape")
    rejects(lnmod.backward, dy.float(), x, sc, mean, rstd, match="dy must be")
    rejects(lnmod.backward, dy, x, t(1, D).expand(B, D), mean, rstd, match="contiguous")
    rejects(lnmod.backward, dy, x, sc, mean, None, match="both")
    rejects(lnmod.backward, dy, x, sc, mean.to(bf), rstd.to(bf), match="float32")
    rejects(lnmod.backward, dy, x, sc, t(B, S - 1, dtype=f32), t(B, S - 1, dtype=f32), match="mean must have shape")
    rejects(lnmod.backward, dy, x, sc, mean, rstd, ws=torch.zeros(8, dtype=torch.uint8), match="bytes")
    rejects(lnmod.backward, dy, x, sc, mean, rstd, ws=torch.zeros(1 << 20, dtype=f32), match="uint8")
    rejects(lnmod.backward, dy, x, sc, mean, rstd, match="GPU")


def test_varlen_rejections():
    T, nseg = 10, 3
    x, dy, sh, sc = t(T, D), t(T, D), t(nseg, D), t(nseg, D)
    cu = torch.tensor([0, 4, 4, 10], dtype=torch.int32)
    rejects(lnmod.forward_varlen, x, sh, sc, cu.long(), match="int32")
    rejects(lnmod.forward_varlen, x, sh, sc, cu.view(2, 2), match="1-D")
    rejects(lnmod.forward_varlen, x, t(nseg + 1, D), sc, cu, match="shift must have shape")
    rejects(lnmod.forward_varlen, t(1, T, D), sh, sc, cu, match="packed")
    rejects(lnmod.forward_varlen, x, sh, sc, cu, match="GPU")
    rejects(lnmod.backward_varlen, dy, x, sc.float(), cu, None, None, match="scale must be")
    rejects(lnmod.backward_varlen, dy, x, sc, cu, t(T + 1, dtype=f32), t(T + 1, dtype=f32), match="mean must have shape")
    rejects(lnmod.backward_varlen, t(T, D + 8), x, sc, cu, None, None, match="dy must have shape")
    rejects(lnmod.backward_varlen, dy, x, sc, cu, None, None, match="GPU")


def test_gated_rejections():
    x, u = t(B, S, D), t(B, S, D)
    g, sh, sc = t(B, D), t(B, D), t(B, D)
    rejects(lnmod.gated_forward, x, t(B, S - 1, D), g, sh, sc, match="u must have shape")
    rejects(lnmod.gated_forward, x, u, t(1, D).expand(B, D), sh, sc, match="contiguous")
    rejects(lnmod.gated_forward, x, u, g.float(), sh, sc, match="gate must be")
    rejects(lnmod.gated_forward, x, u, g, sh, sc, match="GPU")
    mean, rstd = t(B * S, dtype=f32), t(B * S, dtype=f32)
    rejects(lnmod.gated_backward, x, x, x, t(B, S, D + 8), g, sc, mean, rstd, match="u must have shape")
    rejects(lnmod.gated_backward, x, x, x, u, g, sc, mean, t(B * S + 1, dtype=f32), match="rstd must have shape")
    rejects(lnmod.gated_backward, x, x, x, u, g, sc, mean, rstd, match="GPU")
    cu = torch.tensor([0, 4, 12], dtype=torch.int32)
    rejects(lnmod.gated_forward, t(12, D), t(12, D), t(3, D), t(2, D), t(2, D), cu, match="gate must have shape")


def test_qknorm_rejections():
    q, k, w = t(20, 4, D), t(20, 4, D), t(D)
    rejects(lnmod.qknorm_forward, q, t(19, 4, D), w, w, match="k must have shape")      # k with fewer rows than q
    rejects(lnmod.qknorm_forward, q, k, t(D + 8), w, match="wq must have shape")
    rejects(lnmod.qknorm_forward, q, k, w, w.float(), match="wk must be")
    rejects(lnmod.qknorm_forward, q, k.transpose(0, 1).contiguous().transpose(0, 1), w, w, match="contiguous")
    rejects(lnmod.qknorm_forward, q, k, w, w, match="GPU")
    r = t(80, dtype=f32)
    rejects(lnmod.qknorm_backward, q, k, q, t(20, 3, D), w, w, r, r, match="k must have shape")
    rejects(lnmod.qknorm_backward, q, k, q, k, w, w, r, t(79, dtype=f32), match="rstd_k must have shape")
    rejects(lnmod.qknorm_backward, q, k, q, k, w, w, r, r, match="GPU")
