"""ctypes front end of the float64 CPU oracle of the gated-residual + LayerNorm-Modulate
operator (gated_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  The product package never imports this module, and this module imports
nothing from the product package.  The arithmetic lives entirely in gated_oracle.c (its header
states the formulas); this file compiles that source with gcc, hands numpy arrays to it and
shapes the results.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(_HERE, "gated_oracle.c")
LIBRARY = os.path.join(_HERE, "libgated_oracle.so")

QUANT_NONE = 0     # h kept exact (differentiation pins)
QUANT_F32 = 1      # h stored as float32
QUANT_BF16 = 2     # h stored as bfloat16 (float32 first, then bf16, both to nearest even)

_lock = threading.Lock()
_lib = None


def build(force: bool = False, source: str = SOURCE, output: str = LIBRARY) -> str:
    """Compile the C oracle into a shared library with gcc (-O2, no fast-math, OpenMP)."""
    if (not force and os.path.exists(output)
            and os.path.getmtime(output) >= os.path.getmtime(source)):
        return output
    tmp = output + ".tmp.%d" % os.getpid()
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
           "-o", tmp, source, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, output)
    return output


def load(path: str | None = None) -> ctypes.CDLL:
    global _lib
    with _lock:
        if path is None and _lib is not None:
            return _lib
        lib = ctypes.CDLL(path if path is not None else build())
        i64, vp, dbl, cint = ctypes.c_int64, ctypes.c_void_p, ctypes.c_double, ctypes.c_int
        lib.gated_oracle_forward.restype = cint
        lib.gated_oracle_forward.argtypes = [vp, vp, vp, vp, vp, cint, vp, i64, i64, dbl, cint,
                                             vp, vp, vp, vp]
        lib.gated_oracle_backward.restype = cint
        lib.gated_oracle_backward.argtypes = [vp, vp, vp, vp, vp, vp, cint, vp, i64, i64, dbl,
                                              vp, vp, vp, vp, vp]
        if path is None:
            _lib = lib
        return lib


def _carrier(*arrays):
    f32 = all(np.asarray(a).dtype == np.float32 for a in arrays)
    dt = np.float32 if f32 else np.float64
    return [np.ascontiguousarray(a, dtype=dt) for a in arrays], int(f32)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _segments(T: int, cu, B, S):
    if cu is None:
        if B is None or S is None:
            raise ValueError("give either cu or (B, S)")
        cu = np.arange(B + 1, dtype=np.int64) * int(S)
    cu = np.ascontiguousarray(cu, dtype=np.int64)
    if cu.ndim != 1 or cu.size < 1 or cu[0] != 0 or cu[-1] != T:
        raise ValueError("segment offsets must start at 0 and end at the token count")
    return cu


def forward(x, u, gate, shift, scale, eps=1e-6, *, B=None, S=None, cu=None, quant=QUANT_NONE,
            lib=None):
    """h, y, mean, rstd in float64.  x, u: [T, D]; gate, shift, scale: [nseg, D]."""
    x = np.asarray(x)
    T, D = x.shape
    cu = _segments(T, cu, B, S)
    nseg = cu.size - 1
    (x_c, u_c, g_c, sh_c, sc_c), f32 = _carrier(
        x, np.asarray(u).reshape(T, D), np.asarray(gate).reshape(nseg, D),
        np.asarray(shift).reshape(nseg, D), np.asarray(scale).reshape(nseg, D))
    h = np.empty((T, D), dtype=np.float64)
    y = np.empty((T, D), dtype=np.float64)
    mean = np.empty(T, dtype=np.float64)
    rstd = np.empty(T, dtype=np.float64)
    rc = (lib or load()).gated_oracle_forward(_ptr(x_c), _ptr(u_c), _ptr(g_c), _ptr(sh_c),
                                              _ptr(sc_c), f32, _ptr(cu), nseg, D, float(eps),
                                              int(quant), _ptr(h), _ptr(y), _ptr(mean), _ptr(rstd))
    if rc != 0:
        raise RuntimeError("gated_oracle_forward failed with status %d" % rc)
    return h, y, mean, rstd


def backward(dy, dh, h, u, gate, scale, eps=1e-6, *, B=None, S=None, cu=None, lib=None):
    """dx, du [T, D] and dgate, dshift, dscale [nseg, D] in float64 (statistics recomputed from h)."""
    h = np.asarray(h)
    T, D = h.shape
    cu = _segments(T, cu, B, S)
    nseg = cu.size - 1
    (dy_c, dh_c, h_c, u_c, g_c, sc_c), f32 = _carrier(
        np.asarray(dy).reshape(T, D), np.asarray(dh).reshape(T, D), h, np.asarray(u).reshape(T, D),
        np.asarray(gate).reshape(nseg, D), np.asarray(scale).reshape(nseg, D))
    dx = np.empty((T, D), dtype=np.float64)
    du = np.empty((T, D), dtype=np.float64)
    dgate = np.empty((nseg, D), dtype=np.float64)
    dshift = np.empty((nseg, D), dtype=np.float64)
    dscale = np.empty((nseg, D), dtype=np.float64)
    rc = (lib or load()).gated_oracle_backward(_ptr(dy_c), _ptr(dh_c), _ptr(h_c), _ptr(u_c),
                                               _ptr(g_c), _ptr(sc_c), f32, _ptr(cu), nseg, D,
                                               float(eps), _ptr(dx), _ptr(du), _ptr(dgate),
                                               _ptr(dshift), _ptr(dscale))
    if rc != 0:
        raise RuntimeError("gated_oracle_backward failed with status %d" % rc)
    return dx, du, dgate, dshift, dscale
