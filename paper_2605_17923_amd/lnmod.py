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

_HERE = os.path.dirname(os.path.abspath(__file__))
LIBRARY = os.path.join(_HERE, "liblnmod.so")

LNMOD_STATIC_WORKSPACE_BYTES = 64 << 20

EXPORTS = ("lnmod_forward", "lnmod_backward", "lnmod_forward_varlen", "lnmod_backward_varlen",
           "lnmod_backward_static", "lnmod_backward_workspace_bytes", "lnmod_status_string", "lnmod_gated_forward",
           "lnmod_gated_backward", "lnmod_gated_backward_workspace_bytes", "lnmod_qknorm_forward",
           "lnmod_qknorm_backward", "lnmod_qknorm_backward_workspace_bytes")

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
    lib.lnmod_backward_static.restype = cint
    lib.lnmod_backward_static.argtypes = [vp, vp, vp, vp, i64, i64, i64, f32, vp, vp, vp, vp, vp, vp,
                                          cint, cint]
    lib.lnmod_forward_varlen.restype = cint
    lib.lnmod_forward_varlen.argtypes = [vp, vp, vp, vp, i64, i64, i64, f32, vp, vp, vp, vp, cint]
    lib.lnmod_backward_varlen.restype = cint
    lib.lnmod_backward_varlen.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, f32, vp, vp, vp,
                                          vp, vp, vp, vp, sz, cint]
    lib.lnmod_backward_workspace_bytes.restype = sz
    lib.lnmod_backward_workspace_bytes.argtypes = [i64, i64, i64, cint]
    lib.lnmod_status_string.restype = ctypes.c_char_p
    lib.lnmod_status_string.argtypes = [cint]
    lib.lnmod_gated_forward.restype = cint
    lib.lnmod_gated_forward.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, f32, vp,
                                        vp, vp, vp, vp, cint]
    lib.lnmod_gated_backward.restype = cint
    lib.lnmod_gated_backward.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, f32, vp,
                                         vp, vp, vp, vp, vp, vp, vp, vp, sz, cint]
    lib.lnmod_gated_backward_workspace_bytes.restype = sz
    lib.lnmod_gated_backward_workspace_bytes.argtypes = [i64, i64, i64]
    lib.lnmod_qknorm_forward.restype = cint
    lib.lnmod_qknorm_forward.argtypes = [vp, vp, vp, vp, i64, i64, f32, vp, vp, vp, vp, vp, cint]
    lib.lnmod_qknorm_backward.restype = cint
    lib.lnmod_qknorm_backward.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, f32, vp, vp, vp,
                                          vp, vp, vp, vp, vp, sz, cint]
    lib.lnmod_qknorm_backward_workspace_bytes.restype = sz
    lib.lnmod_qknorm_backward_workspace_bytes.argtypes = [i64, i64]
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


def lnmod_backward_static(dy, x, shift, scale, B, S, D, eps, stream, mean, rstd, dx, dshift, dscale,
                          dtype, mod):
    return library().lnmod_backward_static(_p(dy), _p(x), _p(shift), _p(scale), B, S, D, eps, stream,
                                           _p(mean), _p(rstd), _p(dx), _p(dshift), _p(dscale),
                                           dtype, mod)


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




# ---- conveniences: check the tensors, allocate outputs with torch, raise on a non-zero status ---
# The C entry points see addresses only, so a tensor of the wrong shape, element type, layout or
# device would be read out of bounds or misread by the kernels.  Everything a wrapper passes down
# is therefore checked here first; a mismatch raises ValueError and nothing is launched.
def _dtype_code(t):
    import torch
    if t.dtype == torch.bfloat16:
        return LNMOD_BF16
    if t.dtype == torch.float32:
        return LNMOD_F32
    raise ValueError("x must be bfloat16 or float32, got %s" % (t.dtype,))


def _check(status, where):
    if status != LNMOD_OK:
        raise LnmodError(status, where)


class _Args:
    """Collects the tensors of one call.  expect() checks shape, element type and layout at once;
    on_gpu() then checks that all of them sit on one GPU.  The device comes last so that the other
    rejections can be exercised with host tensors."""

    def __init__(self, ref):
        import torch
        if not isinstance(ref, torch.Tensor):
            raise ValueError("x must be a tensor")
        self.ref = ref
        self.seen = []

    def expect(self, name, t, shape, dtype=None):
        import torch
        if not isinstance(t, torch.Tensor):
            raise ValueError("%s must be a tensor" % name)
        if tuple(t.shape) != tuple(shape):
            raise ValueError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
        want = self.ref.dtype if dtype is None else dtype
        if t.dtype != want:
            raise ValueError("%s must be %s, got %s" % (name, want, t.dtype))
        if not t.is_contiguous():
            raise ValueError("%s must be contiguous (dense, last dimension fastest; an expanded or "
                             "sliced view is not)" % name)
        self.seen.append((name, t))

    def expect_pair(self, a_name, a, b_name, b, shape):
        """Two float32 tensors that are given together or not at all (the saved statistics)."""
        import torch
        if (a is None) != (b is None):
            raise ValueError("%s and %s must both be given or both be None" % (a_name, b_name))
        if a is not None:
            self.expect(a_name, a, shape, torch.float32)
            self.expect(b_name, b, shape, torch.float32)

    def expect_cu(self, cu):
        """cu_seqlens: int32 [nseg+1] -> nseg."""
        import torch
        if not isinstance(cu, torch.Tensor) or cu.dim() != 1 or cu.numel() < 1:
            raise ValueError("cu_seqlens must be a 1-D tensor of nseg+1 offsets")
        self.expect("cu_seqlens", cu, cu.shape, torch.int32)
        return cu.numel() - 1

    def expect_workspace(self, ws, need):
        import torch
        if ws is None:
            return
        if not isinstance(ws, torch.Tensor) or ws.dtype != torch.uint8 or ws.dim() != 1 or not ws.is_contiguous():
            raise ValueError("ws must be a dense 1-D uint8 tensor")
        if ws.numel() < need:
            raise ValueError("ws holds %d bytes, %d are needed" % (ws.numel(), need))
        self.seen.append(("ws", ws))

    def on_gpu(self):
        if not self.ref.is_cuda:
            raise ValueError("tensors must be on a GPU (there is no CPU path)")
        for name, t in self.seen:
            if t.device != self.ref.device:
                raise ValueError("%s is on %s, x on %s" % (name, t.device, self.ref.device))


class _on_stream:
    """Work (allocations included) goes to `stream`: None is torch's current stream; a
    torch.cuda.Stream or a raw hipStream_t handle becomes the current stream for the duration,
    so that outputs and the temporary workspace come from that stream's memory pool and are not
    handed to another allocation while the kernels are still queued."""

    def __init__(self, stream):
        import torch
        if stream is None:
            self._ctx = None
        elif isinstance(stream, int):
            self._ctx = torch.cuda.stream(torch.cuda.ExternalStream(stream))
        else:
            self._ctx = torch.cuda.stream(stream)

    def __enter__(self):
        import torch
        if self._ctx is not None:
            self._ctx.__enter__()
        return torch.cuda.current_stream().cuda_stream

    def __exit__(self, *exc):
        if self._ctx is not None:
            self._ctx.__exit__(*exc)
        return False


def _mod_rows(x, shift_or_scale, name):
    """x [B,S,D]; the modulation tensor is [B,D] (per sample) or [B,S,D] (per token)."""
    if x.dim() != 3:
        raise ValueError("x must be [B, S, D], got %s" % (tuple(x.shape),))
    B, S, D = x.shape
    if shift_or_scale.dim() == 3:
        return LNMOD_PER_TOKEN, (B, S, D)
    if shift_or_scale.dim() == 2:
        return LNMOD_PER_SAMPLE, (B, D)
    raise ValueError("%s must be [B, D] or [B, S, D], got %s" % (name, tuple(shift_or_scale.shape)))


def forward(x, shift, scale, eps=1e-6, stream=None):
    """x [B,S,D]; shift, scale [B,D] (per sample) or [B,S,D] (per token) -> y, mean, rstd."""
    import torch
    code = _dtype_code(x)
    mod, mshape = _mod_rows(x, scale, "scale")
    B, S, D = x.shape
    a = _Args(x)
    a.expect("x", x, (B, S, D))
    a.expect("shift", shift, mshape)
    a.expect("scale", scale, mshape)
    a.on_gpu()
    with _on_stream(stream) as handle:
        y = torch.empty_like(x)
        mean = torch.empty(B * S, dtype=torch.float32, device=x.device)
        rstd = torch.empty(B * S, dtype=torch.float32, device=x.device)
        _check(lnmod_forward(x, shift, scale, B, S, D, eps, handle, y, mean, rstd, code, mod),
               "lnmod_forward")
    return y, mean.view(B, S), rstd.view(B, S)


def workspace(B_or_nseg, total_tokens, D, device):
    import torch
    n = lnmod_backward_workspace_bytes(B_or_nseg, total_tokens, D, LNMOD_PER_SAMPLE)
    return torch.empty(max(n, 16), dtype=torch.uint8, device=device)


def backward(dy, x, scale, mean, rstd, eps=1e-6, stream=None, ws=None):
    """-> dx, dshift, dscale (float32 [B,D] per sample; I/O dtype [B,S,D] per token).
    mean = rstd = None: the statistics are formed again from x with eps."""
    import torch
    code = _dtype_code(x)
    mod, mshape = _mod_rows(x, scale, "scale")
    B, S, D = x.shape
    a = _Args(x)
    a.expect("x", x, (B, S, D))
    a.expect("dy", dy, (B, S, D))
    a.expect("scale", scale, mshape)
    # the statistics as forward() returns them ([B, S]) or flat
    if mean is not None and tuple(mean.shape) == (B, S) and mean.is_contiguous():
        mean = mean.view(B * S)
    if rstd is not None and tuple(rstd.shape) == (B, S) and rstd.is_contiguous():
        rstd = rstd.view(B * S)
    a.expect_pair("mean", mean, "rstd", rstd, (B * S,))
    if mod == LNMOD_PER_SAMPLE:
        a.expect_workspace(ws, lnmod_backward_workspace_bytes(B, B * S, D, mod))
    a.on_gpu()
    with _on_stream(stream) as handle:
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
        _check(lnmod_backward(dy, x, None, scale, B, S, D, eps, handle, mean, rstd, dx, dshift,
                              dscale, ws_ptr, ws_bytes, code, mod), "lnmod_backward")
    return dx, dshift, dscale


def _packed(x):
    if x.dim() != 2:
        raise ValueError("x must be packed [T, D], got %s" % (tuple(x.shape),))
    return x.shape


def forward_varlen(x, shift, scale, cu_seqlens, eps=1e-6, stream=None):
    """x [T,D] packed; shift, scale [nseg,D]; cu_seqlens int32 [nseg+1] on the device."""
    import torch
    code = _dtype_code(x)
    T, D = _packed(x)
    a = _Args(x)
    nseg = a.expect_cu(cu_seqlens)
    a.expect("x", x, (T, D))
    a.expect("shift", shift, (nseg, D))
    a.expect("scale", scale, (nseg, D))
    a.on_gpu()
    with _on_stream(stream) as handle:
        y = torch.empty_like(x)
        mean = torch.empty(T, dtype=torch.float32, device=x.device)
        rstd = torch.empty(T, dtype=torch.float32, device=x.device)
        _check(lnmod_forward_varlen(x, shift, scale, cu_seqlens, nseg, T, D, eps, handle, y, mean,
                                    rstd, code), "lnmod_forward_varlen")
    return y, mean, rstd


def backward_varlen(dy, x, scale, cu_seqlens, mean, rstd, eps=1e-6, stream=None, ws=None):
    import torch
    code = _dtype_code(x)
    T, D = _packed(x)
    a = _Args(x)
    nseg = a.expect_cu(cu_seqlens)
    a.expect("x", x, (T, D))
    a.expect("dy", dy, (T, D))
    a.expect("scale", scale, (nseg, D))
    a.expect_pair("mean", mean, "rstd", rstd, (T,))
    a.expect_workspace(ws, lnmod_backward_workspace_bytes(nseg, T, D, LNMOD_PER_SAMPLE))
    a.on_gpu()
    with _on_stream(stream) as handle:
        dx = torch.empty_like(x)
        dshift = torch.empty(nseg, D, dtype=torch.float32, device=x.device)
        dscale = torch.empty(nseg, D, dtype=torch.float32, device=x.device)
        if ws is None:
            ws = workspace(nseg, T, D, x.device)
        _check(lnmod_backward_varlen(dy, x, None, scale, cu_seqlens, nseg, T, D, eps, handle, mean,
                                     rstd, dx, dshift, dscale, ws, ws.numel(), code),
               "lnmod_backward_varlen")
    return dx, dshift, dscale


def gated_workspace(B_or_nseg, total_tokens, D, device):
    import torch
    n = lnmod_gated_backward_workspace_bytes(B_or_nseg, total_tokens, D)
    return torch.empty(max(n, 16), dtype=torch.uint8, device=device)


def _gated_shape(a, x, cu_seqlens):
    """-> (samples or segments, S or T, total tokens, D)."""
    if cu_seqlens is None:
        if x.dim() != 3:
            raise ValueError("x must be [B, S, D] without cu_seqlens, got %s" % (tuple(x.shape),))
        B, S, D = x.shape
        return B, S, B * S, D
    T, D = _packed(x)
    return a.expect_cu(cu_seqlens), T, T, D


def gated_forward(x, u, gate, shift, scale, cu_seqlens=None, eps=1e-6, stream=None):
    """h = x + gate*u (stored), y = LayerNorm-Modulate(h).  x, u: [B,S,D] with gate/shift/scale
    [B,D], or packed [T,D] with cu_seqlens (device int32 [nseg+1]) and [nseg,D] modulation rows.
    -> h, y, mean, rstd."""
    import torch
    code = _dtype_code(x)
    a = _Args(x)
    n, s_or_t, T, D = _gated_shape(a, x, cu_seqlens)
    a.expect("x", x, x.shape)
    a.expect("u", u, x.shape)
    for name, t in (("gate", gate), ("shift", shift), ("scale", scale)):
        a.expect(name, t, (n, D))
    a.on_gpu()
    with _on_stream(stream) as handle:
        h, y = torch.empty_like(x), torch.empty_like(x)
        mean = torch.empty(T, dtype=torch.float32, device=x.device)
        rstd = torch.empty(T, dtype=torch.float32, device=x.device)
        _check(lnmod_gated_forward(x, u, gate, shift, scale, cu_seqlens, n, s_or_t, D, eps, handle,
                                   h, y, mean, rstd, code), "lnmod_gated_forward")
    return h, y, mean, rstd


def gated_backward(dy, dh, h, u, gate, scale, mean, rstd, cu_seqlens=None, eps=1e-6, stream=None,
                   ws=None):
    """-> dx, du (I/O dtype) and dgate, dshift, dscale (float32 [B,D] / [nseg,D])."""
    import torch
    code = _dtype_code(h)
    a = _Args(h)
    n, s_or_t, T, D = _gated_shape(a, h, cu_seqlens)
    a.expect("h", h, h.shape)
    for name, t in (("dy", dy), ("dh", dh), ("u", u)):
        a.expect(name, t, h.shape)
    a.expect("gate", gate, (n, D))
    a.expect("scale", scale, (n, D))
    a.expect("mean", mean, (T,), torch.float32)
    a.expect("rstd", rstd, (T,), torch.float32)
    a.expect_workspace(ws, lnmod_gated_backward_workspace_bytes(n, T, D))
    a.on_gpu()
    with _on_stream(stream) as handle:
        dx, du = torch.empty_like(h), torch.empty_like(h)
        dgate = torch.empty(n, D, dtype=torch.float32, device=h.device)
        dshift = torch.empty(n, D, dtype=torch.float32, device=h.device)
        dscale = torch.empty(n, D, dtype=torch.float32, device=h.device)
        if ws is None:
            ws = gated_workspace(n, T, D, h.device)
        _check(lnmod_gated_backward(dy, dh, h, u, gate, scale, cu_seqlens, n, s_or_t, D, eps, handle,
                                    mean, rstd, dx, du, dgate, dshift, dscale, ws, ws.numel(), code),
               "lnmod_gated_backward")
    return dx, du, dgate, dshift, dscale


def _qk_rows(q):
    if q.dim() < 1:
        raise ValueError("q must be [..., D]")
    D = q.shape[-1]
    return q.numel() // max(D, 1), D


def qknorm_forward(q, k, wq, wk, eps=1e-6, stream=None):
    """RMS normalisation with weight of q and k ([..., D], same shape) in one launch
    -> q_out, k_out, rstd_q, rstd_k (float32, one per row)."""
    import torch
    code = _dtype_code(q)
    N, D = _qk_rows(q)
    a = _Args(q)
    a.expect("q", q, q.shape)
    a.expect("k", k, q.shape)
    a.expect("wq", wq, (D,))
    a.expect("wk", wk, (D,))
    a.on_gpu()
    with _on_stream(stream) as handle:
        q_out, k_out = torch.empty_like(q), torch.empty_like(k)
        rq = torch.empty(N, dtype=torch.float32, device=q.device)
        rk = torch.empty(N, dtype=torch.float32, device=q.device)
        _check(lnmod_qknorm_forward(q, k, wq, wk, N, D, eps, handle, q_out, k_out, rq, rk, code),
               "lnmod_qknorm_forward")
    return q_out, k_out, rq, rk


def qknorm_backward(dq_out, dk_out, q, k, wq, wk, rstd_q, rstd_k, eps=1e-6, stream=None, ws=None):
    """-> dq, dk (I/O dtype) and dwq, dwk (float32 [D])."""
    import torch
    code = _dtype_code(q)
    N, D = _qk_rows(q)
    a = _Args(q)
    a.expect("q", q, q.shape)
    for name, t in (("k", k), ("dq_out", dq_out), ("dk_out", dk_out)):
        a.expect(name, t, q.shape)
    a.expect("wq", wq, (D,))
    a.expect("wk", wk, (D,))
    a.expect("rstd_q", rstd_q, (N,), torch.float32)
    a.expect("rstd_k", rstd_k, (N,), torch.float32)
    need = lnmod_qknorm_backward_workspace_bytes(N, D)
    a.expect_workspace(ws, need)
    a.on_gpu()
    with _on_stream(stream) as handle:
        dq, dk = torch.empty_like(q), torch.empty_like(k)
        dwq = torch.empty(D, dtype=torch.float32, device=q.device)
        dwk = torch.empty(D, dtype=torch.float32, device=q.device)
        if ws is None:
            ws = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
        _check(lnmod_qknorm_backward(dq_out, dk_out, q, k, wq, wk, N, D, eps, handle, rstd_q, rstd_k,
                                     dq, dk, dwq, dwk, ws, ws.numel(), code), "lnmod_qknorm_backward")
    return dq, dk, dwq, dwk
