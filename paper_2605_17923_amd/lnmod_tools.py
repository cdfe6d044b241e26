"""Thin Python binding of liblnmod_tools.so (the C ABI in include/lnmod_tools.h): bandwidth
references, the unfused comparators and the operator calls that take their launch shape as an
argument.  Used by bench.py and the tests of the launch shapes; no caller of the operators needs
it.  Argument marshalling only; without the built library every call raises.
"""
from __future__ import annotations

import ctypes
import os

from .lnmod import _p

_HERE = os.path.dirname(os.path.abspath(__file__))
LIBRARY = os.path.join(_HERE, "liblnmod_tools.so")

EXPORTS = ("lnmod_copy", "lnmod_stream_probe", "lnmod_unfused_forward", "lnmod_gate_residual",
           "lnmod_table_shape", "lnmod_forward_shaped", "lnmod_backward_shaped",
           "lnmod_backward_workspace_bytes_shaped", "lnmod_describe_launch")

# lnmod_family of include/lnmod_tools.h
(LNMOD_FAMILY_FORWARD, LNMOD_FAMILY_BACKWARD, LNMOD_FAMILY_BACKWARD_RECOMPUTE,
 LNMOD_FAMILY_TOKEN_FORWARD, LNMOD_FAMILY_TOKEN_BACKWARD, LNMOD_FAMILY_GATED_FORWARD,
 LNMOD_FAMILY_GATED_BACKWARD, LNMOD_FAMILY_QKNORM_FORWARD, LNMOD_FAMILY_QKNORM_BACKWARD) = range(9)
LNMOD_FAMILIES = 9

# read/write mixtures lnmod_stream_probe is compiled for
PROBE_MIXTURES = ((1, 0), (0, 1), (1, 1), (2, 1), (2, 2), (3, 1), (3, 3), (4, 2))

_lib = None


def library() -> ctypes.CDLL:
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIBRARY):
        raise RuntimeError("liblnmod_tools.so is not built (run `python -m paper_2605_17923_amd.build` "
                           "or __graft_entry__.build())")
    lib = ctypes.CDLL(LIBRARY)
    vp, i64, f32, cint, sz = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_float, ctypes.c_int,
                              ctypes.c_size_t)
    pint = ctypes.POINTER(cint)
    pvp = ctypes.POINTER(vp)
    lib.lnmod_copy.restype = cint
    lib.lnmod_copy.argtypes = [vp, vp, sz, vp]
    lib.lnmod_stream_probe.restype = cint
    lib.lnmod_stream_probe.argtypes = [pvp, cint, pvp, cint, sz, cint, cint, cint, vp]
    lib.lnmod_unfused_forward.restype = cint
    lib.lnmod_unfused_forward.argtypes = [vp, vp, vp, i64, i64, i64, f32, vp, vp, vp, vp, vp, cint]
    lib.lnmod_gate_residual.restype = cint
    lib.lnmod_gate_residual.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp, cint]
    lib.lnmod_table_shape.restype = cint
    lib.lnmod_table_shape.argtypes = [cint, i64, cint, i64, pint]
    lib.lnmod_forward_shaped.restype = cint
    lib.lnmod_forward_shaped.argtypes = [pint, vp, vp, vp, vp, i64, i64, i64, f32, vp, vp, vp, vp, cint, cint]
    lib.lnmod_backward_shaped.restype = cint
    lib.lnmod_backward_shaped.argtypes = [pint, vp, vp, vp, vp, i64, i64, i64, f32, vp, vp, vp, vp, vp, vp,
                                          vp, sz, cint, cint]
    lib.lnmod_backward_workspace_bytes_shaped.restype = sz
    lib.lnmod_backward_workspace_bytes_shaped.argtypes = [pint, i64, i64, i64, cint]
    lib.lnmod_describe_launch.restype = cint
    lib.lnmod_describe_launch.argtypes = [cint, pint, i64, i64, cint, i64, cint, cint, cint, ctypes.c_char_p, sz]
    _lib = lib
    return lib


def _shape(shape):
    """(K, VPL, R, per_cu[, clusters, interleave, flat]) -> int[7], None -> NULL (the table's entry)."""
    if shape is None:
        return None
    vals = [int(v) for v in shape] + [0, 0, 0]
    return (ctypes.c_int * 7)(*vals[:7])


def _ptr_array(ts):
    arr = (ctypes.c_void_p * max(len(ts), 1))()
    for i, t in enumerate(ts):
        arr[i] = _p(t)
    return arr


def lnmod_copy(src, dst, nbytes, stream):
    return library().lnmod_copy(_p(src), _p(dst), nbytes, stream)


def lnmod_stream_probe(inputs, outputs, nbytes, stream, writes=None, launch=(0, 0, 0)):
    """inputs: tensors read; outputs: tensors written (for a read-only probe pass one tensor of at
    least 1 KB and writes=0).  launch = (blocks, waves, vecs), zeros for the mixture's default."""
    nw = len(outputs) if writes is None else writes
    return library().lnmod_stream_probe(_ptr_array(inputs), len(inputs), _ptr_array(outputs), nw, nbytes,
                                        launch[0], launch[1], launch[2], stream)


def lnmod_unfused_forward(x, shift, scale, B, S, D, eps, stream, xhat_tmp, y, mean, rstd, dtype):
    return library().lnmod_unfused_forward(_p(x), _p(shift), _p(scale), B, S, D, eps, stream,
                                           _p(xhat_tmp), _p(y), _p(mean), _p(rstd), dtype)


def lnmod_gate_residual(x, u, gate, B, S, D, stream, h, dtype):
    return library().lnmod_gate_residual(_p(x), _p(u), _p(gate), B, S, D, stream, _p(h), dtype)


def lnmod_table_shape(family, D, dtype, tokens=0):
    """Returns (status, (K, VPL, R, per_cu))."""
    buf = (ctypes.c_int * 4)()
    st = library().lnmod_table_shape(family, D, dtype, tokens, buf)
    return st, tuple(buf)


def lnmod_forward_shaped(shape, x, shift, scale, cu_seqlens, B_or_nseg, S_or_T, D, eps, stream, y, mean,
                         rstd, dtype, mod):
    return library().lnmod_forward_shaped(_shape(shape), _p(x), _p(shift), _p(scale), _p(cu_seqlens),
                                          B_or_nseg, S_or_T, D, eps, stream, _p(y), _p(mean), _p(rstd),
                                          dtype, mod)


def lnmod_backward_shaped(shape, dy, x, scale, cu_seqlens, B_or_nseg, S_or_T, D, eps, stream, mean, rstd,
                          dx, dshift, dscale, workspace, workspace_bytes, dtype, mod):
    return library().lnmod_backward_shaped(_shape(shape), _p(dy), _p(x), _p(scale), _p(cu_seqlens),
                                           B_or_nseg, S_or_T, D, eps, stream, _p(mean), _p(rstd), _p(dx),
                                           _p(dshift), _p(dscale), _p(workspace), workspace_bytes, dtype,
                                           mod)


def lnmod_backward_workspace_bytes_shaped(shape, B_or_nseg, total_tokens, D, mod):
    return int(library().lnmod_backward_workspace_bytes_shaped(_shape(shape), B_or_nseg, total_tokens, D, mod))


def lnmod_describe_launch(backward, shape, B_or_nseg, S_or_T, varlen, D, dtype, mod, recompute=False):
    """The kernel instantiations and grids the call launches, as text ('' for invalid arguments)."""
    buf = ctypes.create_string_buffer(512)
    library().lnmod_describe_launch(int(bool(backward)), _shape(shape), B_or_nseg, S_or_T, int(bool(varlen)), D,
                                    dtype, mod, int(bool(recompute)), buf, len(buf))
    return buf.value.decode()
