"""Thin Python binding of liblnmod.so (the C ABI in include/lnmod.h).

Argument marshalling only: every arithmetic step runs in the gfx950 kernels.  PyTorch is used
for device memory and streams, nothing else.  The lnmod_* functions mirror the C entry points
one to one (tensors or raw integer addresses for pointers); forward()/backward() and their
varlen forms additionally allocate the outputs and the workspace with torch.

There is no CPU fallback: if the shared library is missing, every call raises.
"""
from __future__ import annotations

import ctypes
import os

LNMOD_OK, LNMOD_EINVAL, LNMOD_EUNSUPPORTED, LNMOD_EALIGN, LNMOD_EWORKSPACE, LNMOD_ELAUNCH = range(6)
LNMOD_BF16, LNMOD_F32 = 0, 1
LNMOD_PER_SAMPLE, LNMOD_PER_TOKEN = 0, 1
LNMOD_PROBE_ADD, LNMOD_PROBE_READ, LNMOD_PROBE_WRITE = 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
LIBRARY = os.path.join(_HERE, "liblnmod.so")

EXPORTS = ("lnmod_forward", "lnmod_backward", "lnmod_forward_varlen", "lnmod_backward_varlen",
           "lnmod_backward_workspace_bytes", "lnmod_status_string", "lnmod_unfused_forward",
           "lnmod_copy", "lnmod_stream_probe", "lnmod_gated_forward", "lnmod_gated_backward",
           "lnmod_gated_backward_workspace_bytes", "lnmod_gate_residual", "lnmod_qknorm_forward",
           "lnmod_qknorm_backward", "lnmod_qknorm_backward_workspace_bytes")
TUNING_EXPORTS = ("lnmod_tuning_set_shape", "lnmod_tuning_table_shape")

# lnmod_tune_family of include/lnmod_tuning.h
(LNMOD_TUNE_FORWARD, LNMOD_TUNE_BACKWARD, LNMOD_TUNE_BACKWARD_RECOMPUTE, LNMOD_TUNE_TOKEN_FORWARD,
 LNMOD_TUNE_TOKEN_BACKWARD, LNMOD_TUNE_GATED_FORWARD, LNMOD_TUNE_GATED_BACKWARD,
 LNMOD_TUNE_QKNORM_FORWARD, LNMOD_TUNE_QKNORM_BACKWARD) = range(9)
LNMOD_TUNE_FAMILIES = 9

_lib = None


class LnmodError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (status %d)" % (where, lnmod_status_string(status), status))


def library() -> ctypes.CDLL:
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIBRARY):
        raise RuntimeError("liblnmod.so is not built (run `python -m paper_2605_17923_amd.build` "
                           "or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(LIBRARY)
    vp, i64, f32, cint, sz = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_float, ctypes.c_int,
                              ctypes.c_size_t)
    lib.lnmod_forward.restype = cint
    lib.lnmod_forward.argtypes = [vp, vp, vp, i64, i64, i64, f32, vp, vp, vp, vp, cint, cint]
    lib.lnmod_backward.restype = cint
    lib.lnmod_backward.argtypes = [vp, vp, vp, vp, i64, i64, i64, f32, vp, vp, vp, vp, vp, vp,
                                   vp, sz, cint, cint]
    lib.lnmod_forward_varlen.restype = cint
    lib.lnmod_forward_varlen.argtypes = [vp, vp, vp, vp, i64, i64, i64, f32, vp, vp, vp, vp, cint]
    lib.lnmod_backward_varlen.restype = cint
    lib.lnmod_backward_varlen.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, f32, vp, vp, vp,
                                          vp, vp, vp, vp, sz, cint]
    lib.lnmod_backward_workspace_bytes.restype = sz
    lib.lnmod_backward_workspace_bytes.argtypes = [i64, i64, i64, cint]
    lib.lnmod_status_string.restype = ctypes.c_char_p
    lib.lnmod_status_string.argtypes = [cint]
    lib.lnmod_unfused_forward.restype = cint
    lib.lnmod_unfused_forward.argtypes = [vp, vp, vp, i64, i64, i64, f32, vp, vp, vp, vp, vp, cint]
    lib.lnmod_copy.restype = cint
    lib.lnmod_copy.argtypes = [vp, vp, sz, vp]
    lib.lnmod_stream_probe.restype = cint
    lib.lnmod_stream_probe.argtypes = [vp, vp, vp, sz, cint, vp]
    lib.lnmod_gated_forward.restype = cint
    lib.lnmod_gated_forward.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, f32, vp,
                                        vp, vp, vp, vp, cint]
    lib.lnmod_gated_backward.restype = cint
    lib.lnmod_gated_backward.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, f32, vp,
                                         vp, vp, vp, vp, vp, vp, vp, vp, sz, cint]
    lib.lnmod_gated_backward_workspace_bytes.restype = sz
    lib.lnmod_gated_backward_workspace_bytes.argtypes = [i64, i64, i64]
    lib.lnmod_gate_residual.restype = cint
    lib.lnmod_gate_residual.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp, cint]
    lib.lnmod_qknorm_forward.restype = cint
    lib.lnmod_qknorm_forward.argtypes = [vp, vp, vp, vp, i64, i64, f32, vp, vp, vp, vp, vp, cint]
    lib.lnmod_qknorm_backward.restype = cint
    lib.lnmod_qknorm_backward.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, f32, vp, vp, vp,
                                          vp, vp, vp, vp, vp, sz, cint]
    lib.lnmod_qknorm_backward_workspace_bytes.restype = sz
    lib.lnmod_qknorm_backward_workspace_bytes.argtypes = [i64, i64]
    lib.lnmod_tuning_set_shape.restype = cint
    lib.lnmod_tuning_set_shape.argtypes = [cint, cint, cint, cint, cint]
    lib.lnmod_tuning_table_shape.restype = cint
    lib.lnmod_tuning_table_shape.argtypes = [cint, i64, cint, ctypes.POINTER(cint)]
    _lib = lib
    return lib


def _p(t):
    """Device address of a tensor, an integer address as is, None as NULL."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream_handle(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


# ---- one-to-one mirrors of the C entry points (return the status code) -------------------------
def lnmod_forward(x, shift, scale, B, S, D, eps, stream, y, mean, rstd, dtype, mod):
    return library().lnmod_forward(_p(x), _p(shift), _p(scale), B, S, D, eps, stream,
                                   _p(y), _p(mean), _p(rstd), dtype, mod)


def lnmod_backward(dy, x, shift, scale, B, S, D, eps, stream, mean, rstd, dx, dshift, dscale,
                   workspace, workspace_bytes, dtype, mod):
    return library().lnmod_backward(_p(dy), _p(x), _p(shift), _p(scale), B, S, D, eps, stream,
                                    _p(mean), _p(rstd), _p(dx), _p(dshift), _p(dscale),
                                    _p(workspace), workspace_bytes, dtype, mod)


def lnmod_forward_varlen(x, shift, scale, cu_seqlens, nseg, T, D, eps, stream, y, mean, rstd, dtype):
    return library().lnmod_forward_varlen(_p(x), _p(shift), _p(scale), _p(cu_seqlens), nseg, T, D,
                                          eps, stream, _p(y), _p(mean), _p(rstd), dtype)


def lnmod_backward_varlen(dy, x, shift, scale, cu_seqlens, nseg, T, D, eps, stream, mean, rstd,
                          dx, dshift, dscale, workspace, workspace_bytes, dtype):
    return library().lnmod_backward_varlen(_p(dy), _p(x), _p(shift), _p(scale), _p(cu_seqlens),
                                           nseg, T, D, eps, stream, _p(mean), _p(rstd), _p(dx),
                                           _p(dshift), _p(dscale), _p(workspace), workspace_bytes,
                                           dtype)


def lnmod_backward_workspace_bytes(B_or_nseg, total_tokens, D, mod):
    return int(library().lnmod_backward_workspace_bytes(B_or_nseg, total_tokens, D, mod))


def lnmod_status_string(status):
    return library().lnmod_status_string(int(status)).decode()


def lnmod_unfused_forward(x, shift, scale, B, S, D, eps, stream, xhat_tmp, y, mean, rstd, dtype):
    return library().lnmod_unfused_forward(_p(x), _p(shift), _p(scale), B, S, D, eps, stream,
                                           _p(xhat_tmp), _p(y), _p(mean), _p(rstd), dtype)


def lnmod_copy(src, dst, nbytes, stream):
    return library().lnmod_copy(_p(src), _p(dst), nbytes, stream)


def lnmod_stream_probe(a, b, c, nbytes, mode, stream):
    return library().lnmod_stream_probe(_p(a), _p(b), _p(c), nbytes, mode, stream)


def lnmod_gated_forward(x, u, gate, shift, scale, cu_seqlens, B_or_nseg, S_or_T, D, eps, stream,
                        h, y, mean, rstd, dtype):
    return library().lnmod_gated_forward(_p(x), _p(u), _p(gate), _p(shift), _p(scale),
                                         _p(cu_seqlens), B_or_nseg, S_or_T, D, eps, stream,
                                         _p(h), _p(y), _p(mean), _p(rstd), dtype)


def lnmod_gated_backward(dy, dh, h, u, gate, scale, cu_seqlens, B_or_nseg, S_or_T, D, eps, stream,
                         mean, rstd, dx, du, dgate, dshift, dscale, workspace, workspace_bytes,
                         dtype):
    return library().lnmod_gated_backward(_p(dy), _p(dh), _p(h), _p(u), _p(gate), _p(scale),
                                          _p(cu_seqlens), B_or_nseg, S_or_T, D, eps, stream,
                                          _p(mean), _p(rstd), _p(dx), _p(du), _p(dgate),
                                          _p(dshift), _p(dscale), _p(workspace), workspace_bytes,
                                          dtype)


def lnmod_gated_backward_workspace_bytes(B_or_nseg, total_tokens, D):
    return int(library().lnmod_gated_backward_workspace_bytes(B_or_nseg, total_tokens, D))


def lnmod_gate_residual(x, u, gate, B, S, D, stream, h, dtype):
    return library().lnmod_gate_residual(_p(x), _p(u), _p(gate), B, S, D, stream, _p(h), dtype)


def lnmod_qknorm_forward(q, k, wq, wk, N, D, eps, stream, q_out, k_out, rstd_q, rstd_k, dtype):
    return library().lnmod_qknorm_forward(_p(q), _p(k), _p(wq), _p(wk), N, D, eps, stream,
                                          _p(q_out), _p(k_out), _p(rstd_q), _p(rstd_k), dtype)


def lnmod_qknorm_backward(dq_out, dk_out, q, k, wq, wk, N, D, eps, stream, rstd_q, rstd_k, dq, dk,
                          dwq, dwk, workspace, workspace_bytes, dtype):
    return library().lnmod_qknorm_backward(_p(dq_out), _p(dk_out), _p(q), _p(k), _p(wq), _p(wk),
                                           N, D, eps, stream, _p(rstd_q), _p(rstd_k), _p(dq),
                                           _p(dk), _p(dwq), _p(dwk), _p(workspace),
                                           workspace_bytes, dtype)


def lnmod_qknorm_backward_workspace_bytes(N, D):
    return int(library().lnmod_qknorm_backward_workspace_bytes(N, D))


# ---- conveniences: allocate outputs with torch, raise on a non-zero status ----------------------
def lnmod_tuning_set_shape(family, K, VPL, R, per_cu):
    return library().lnmod_tuning_set_shape(family, K, VPL, R, per_cu)


def lnmod_tuning_table_shape(family, D, dtype, out=None):
    """Returns (status, (K, VPL, R, per_cu)); `out`, if given, is a ctypes int array of 4."""
    buf = out if out is not None else (ctypes.c_int * 4)()
    st = library().lnmod_tuning_table_shape(family, D, dtype, buf)
    return st, tuple(buf)


def _dtype_code(t):
    import torch
    if t.dtype == torch.bfloat16:
        return LNMOD_BF16
    if t.dtype == torch.float32:
        return LNMOD_F32
    raise TypeError("x must be bfloat16 or float32")


def _check(status, where):
    if status != LNMOD_OK:
        raise LnmodError(status, where)


def forward(x, shift, scale, eps=1e-6, stream=None):
    """x [B,S,D]; shift, scale [B,D] (per sample) or [B,S,D] (per token) -> y, mean, rstd."""
    import torch
    B, S, D = x.shape
    mod = LNMOD_PER_TOKEN if shift.dim() == 3 else LNMOD_PER_SAMPLE
    y = torch.empty_like(x)
    mean = torch.empty(B * S, dtype=torch.float32, device=x.device)
    rstd = torch.empty(B * S, dtype=torch.float32, device=x.device)
    _check(lnmod_forward(x, shift, scale, B, S, D, eps, _stream_handle(stream), y, mean, rstd,
                         _dtype_code(x), mod), "lnmod_forward")
    return y, mean.view(B, S), rstd.view(B, S)


def workspace(B_or_nseg, total_tokens, D, device):
    import torch
    n = lnmod_backward_workspace_bytes(B_or_nseg, total_tokens, D, LNMOD_PER_SAMPLE)
    return torch.empty(max(n, 16), dtype=torch.uint8, device=device)


def backward(dy, x, scale, mean, rstd, eps=1e-6, stream=None, ws=None):
    """-> dx, dshift, dscale (float32 [B,D] per sample; I/O dtype [B,S,D] per token).
    mean = rstd = None: the statistics are formed again from x with eps."""
    import torch
    B, S, D = x.shape
    mod = LNMOD_PER_TOKEN if scale.dim() == 3 else LNMOD_PER_SAMPLE
    dx = torch.empty_like(x)
    if mod == LNMOD_PER_TOKEN:
        dshift, dscale = torch.empty_like(x), torch.empty_like(x)
        ws_ptr, ws_bytes = None, 0
    else:
        dshift = torch.empty(B, D, dtype=torch.float32, device=x.device)
        dscale = torch.empty(B, D, dtype=torch.float32, device=x.device)
        if ws is None:
            ws = workspace(B, B * S, D, x.device)
        ws_ptr, ws_bytes = ws, ws.numel()
    _check(lnmod_backward(dy, x, None, scale, B, S, D, eps, _stream_handle(stream), mean, rstd,
                          dx, dshift, dscale, ws_ptr, ws_bytes, _dtype_code(x), mod),
           "lnmod_backward")
    return dx, dshift, dscale


def forward_varlen(x, shift, scale, cu_seqlens, eps=1e-6, stream=None):
    """x [T,D] packed; shift, scale [nseg,D]; cu_seqlens int32 [nseg+1] on the device."""
    import torch
    T, D = x.shape
    nseg = cu_seqlens.numel() - 1
    y = torch.empty_like(x)
    mean = torch.empty(T, dtype=torch.float32, device=x.device)
    rstd = torch.empty(T, dtype=torch.float32, device=x.device)
    _check(lnmod_forward_varlen(x, shift, scale, cu_seqlens, nseg, T, D, eps,
                                _stream_handle(stream), y, mean, rstd, _dtype_code(x)),
           "lnmod_forward_varlen")
    return y, mean, rstd


def backward_varlen(dy, x, scale, cu_seqlens, mean, rstd, eps=1e-6, stream=None, ws=None):
    import torch
    T, D = x.shape
    nseg = cu_seqlens.numel() - 1
    dx = torch.empty_like(x)
    dshift = torch.empty(nseg, D, dtype=torch.float32, device=x.device)
    dscale = torch.empty(nseg, D, dtype=torch.float32, device=x.device)
    if ws is None:
        ws = workspace(nseg, T, D, x.device)
    _check(lnmod_backward_varlen(dy, x, None, scale, cu_seqlens, nseg, T, D, eps,
                                 _stream_handle(stream), mean, rstd, dx, dshift, dscale, ws,
                                 ws.numel(), _dtype_code(x)), "lnmod_backward_varlen")
    return dx, dshift, dscale


def gated_workspace(B_or_nseg, total_tokens, D, device):
    import torch
    n = lnmod_gated_backward_workspace_bytes(B_or_nseg, total_tokens, D)
    return torch.empty(max(n, 16), dtype=torch.uint8, device=device)


def _gated_shape(x, cu_seqlens):
    if cu_seqlens is None:
        B, S, D = x.shape
        return B, S, B * S, D
    T, D = x.shape
    return cu_seqlens.numel() - 1, T, T, D


def gated_forward(x, u, gate, shift, scale, cu_seqlens=None, eps=1e-6, stream=None):
    """h = x + gate*u (stored), y = LayerNorm-Modulate(h).  x, u: [B,S,D] with gate/shift/scale
    [B,D], or packed [T,D] with cu_seqlens (device int32 [nseg+1]) and [nseg,D] modulation rows.
    -> h, y, mean, rstd."""
    import torch
    n, s_or_t, T, D = _gated_shape(x, cu_seqlens)
    h, y = torch.empty_like(x), torch.empty_like(x)
    mean = torch.empty(T, dtype=torch.float32, device=x.device)
    rstd = torch.empty(T, dtype=torch.float32, device=x.device)
    _check(lnmod_gated_forward(x, u, gate, shift, scale, cu_seqlens, n, s_or_t, D, eps,
                               _stream_handle(stream), h, y, mean, rstd, _dtype_code(x)),
           "lnmod_gated_forward")
    return h, y, mean, rstd


def gated_backward(dy, dh, h, u, gate, scale, mean, rstd, cu_seqlens=None, eps=1e-6, stream=None,
                   ws=None):
    """-> dx, du (I/O dtype) and dgate, dshift, dscale (float32 [B,D] / [nseg,D])."""
    import torch
    n, s_or_t, T, D = _gated_shape(h, cu_seqlens)
    dx, du = torch.empty_like(h), torch.empty_like(h)
    dgate = torch.empty(n, D, dtype=torch.float32, device=h.device)
    dshift = torch.empty(n, D, dtype=torch.float32, device=h.device)
    dscale = torch.empty(n, D, dtype=torch.float32, device=h.device)
    if ws is None:
        ws = gated_workspace(n, T, D, h.device)
    _check(lnmod_gated_backward(dy, dh, h, u, gate, scale, cu_seqlens, n, s_or_t, D, eps,
                                _stream_handle(stream), mean, rstd, dx, du, dgate, dshift, dscale,
                                ws, ws.numel(), _dtype_code(h)), "lnmod_gated_backward")
    return dx, du, dgate, dshift, dscale


def qknorm_forward(q, k, wq, wk, eps=1e-6, stream=None):
    """RMS normalisation with weight of q and k ([..., D], same shape) in one launch
    -> q_out, k_out, rstd_q, rstd_k (float32, one per row)."""
    import torch
    D = q.shape[-1]
    N = q.numel() // D
    q_out, k_out = torch.empty_like(q), torch.empty_like(k)
    rq = torch.empty(N, dtype=torch.float32, device=q.device)
    rk = torch.empty(N, dtype=torch.float32, device=q.device)
    _check(lnmod_qknorm_forward(q, k, wq, wk, N, D, eps, _stream_handle(stream), q_out, k_out, rq, rk,
                                _dtype_code(q)), "lnmod_qknorm_forward")
    return q_out, k_out, rq, rk


def qknorm_backward(dq_out, dk_out, q, k, wq, wk, rstd_q, rstd_k, eps=1e-6, stream=None, ws=None):
    """-> dq, dk (I/O dtype) and dwq, dwk (float32 [D])."""
    import torch
    D = q.shape[-1]
    N = q.numel() // D
    dq, dk = torch.empty_like(q), torch.empty_like(k)
    dwq = torch.empty(D, dtype=torch.float32, device=q.device)
    dwk = torch.empty(D, dtype=torch.float32, device=q.device)
    if ws is None:
        ws = torch.empty(max(lnmod_qknorm_backward_workspace_bytes(N, D), 16), dtype=torch.uint8,
                         device=q.device)
    _check(lnmod_qknorm_backward(dq_out, dk_out, q, k, wq, wk, N, D, eps, _stream_handle(stream),
                                 rstd_q, rstd_k, dq, dk, dwq, dwk, ws, ws.numel(), _dtype_code(q)),
           "lnmod_qknorm_backward")
    return dq, dk, dwq, dwk
