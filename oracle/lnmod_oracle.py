"""ctypes front end of the float64 CPU oracle (lnmod_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  The product package never imports this module, and this module imports
nothing from the product package.

The arithmetic lives entirely in lnmod_oracle.c (see its header for the formulas and the
passage of the paper, Sec. 3.3, they restate).  This file only compiles that source with gcc,
hands numpy arrays to it and shapes the results.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(_HERE, "lnmod_oracle.c")
LIBRARY = os.path.join(_HERE, "liblnmod_oracle.so")

PER_SEGMENT = 0
PER_TOKEN = 1

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
    """Load (building first if needed) the oracle library and declare its prototypes."""
    global _lib
    with _lock:
        if path is None and _lib is not None:
            return _lib
        lib = ctypes.CDLL(path if path is not None else build())
        i64, vp, dbl, cint = ctypes.c_int64, ctypes.c_void_p, ctypes.c_double, ctypes.c_int
        lib.lnmod_oracle_forward.restype = cint
        lib.lnmod_oracle_forward.argtypes = [vp, vp, vp, cint, vp, i64, i64, dbl, cint,
                                             vp, vp, vp]
        lib.lnmod_oracle_backward.restype = cint
        lib.lnmod_oracle_backward.argtypes = [vp, vp, vp, cint, vp, i64, i64, dbl, cint,
                                              vp, vp, vp]
        lib.lnmod_oracle_num_threads.restype = cint
        lib.lnmod_oracle_num_threads.argtypes = []
        lib.lnmod_oracle_set_num_threads.restype = None
        lib.lnmod_oracle_set_num_threads.argtypes = [cint]
        if path is None:
            _lib = lib
        return lib


def num_threads() -> int:
    return int(load().lnmod_oracle_num_threads())


def set_num_threads(n: int) -> None:
    load().lnmod_oracle_set_num_threads(int(n))


def _carrier(*arrays):
    """All inputs as C-contiguous arrays of one carrier type: float32 if every input already
    is float32 (exact carrier of bf16/fp32 data), else float64."""
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


def forward(x, shift, scale, eps=1e-6, *, B=None, S=None, cu=None, mod=PER_SEGMENT, lib=None):
    """y, mean, rstd of LayerNorm-Modulate in float64.

    x: [T, D] tokens (T = B*S for a fixed-length batch).  Either (B, S) or cu (token offsets
    of the segments, length nseg+1) says which modulation row a token uses.
    shift, scale: [nseg, D] (mod=PER_SEGMENT) or [T, D] (mod=PER_TOKEN).
    """
    x = np.asarray(x)
    T, D = x.shape
    cu = _segments(T, cu, B, S)
    nseg = cu.size - 1
    rows = T if mod == PER_TOKEN else nseg
    (x_c, sh_c, sc_c), f32 = _carrier(x, np.asarray(shift).reshape(rows, D),
                                      np.asarray(scale).reshape(rows, D))
    y = np.empty((T, D), dtype=np.float64)
    mean = np.empty(T, dtype=np.float64)
    rstd = np.empty(T, dtype=np.float64)
    rc = (lib or load()).lnmod_oracle_forward(_ptr(x_c), _ptr(sh_c), _ptr(sc_c), f32, _ptr(cu),
                                              nseg, D, float(eps), int(mod),
                                              _ptr(y), _ptr(mean), _ptr(rstd))
    if rc != 0:
        raise RuntimeError("lnmod_oracle_forward failed with status %d" % rc)
    return y, mean, rstd


def backward(dy, x, scale, eps=1e-6, *, B=None, S=None, cu=None, mod=PER_SEGMENT, lib=None):
    """dx, dshift, dscale of LayerNorm-Modulate in float64 (statistics recomputed from x).

    dshift, dscale: [nseg, D] (mod=PER_SEGMENT) or [T, D] (mod=PER_TOKEN).
    """
    x = np.asarray(x)
    T, D = x.shape
    cu = _segments(T, cu, B, S)
    nseg = cu.size - 1
    rows = T if mod == PER_TOKEN else nseg
    (dy_c, x_c, sc_c), f32 = _carrier(np.asarray(dy).reshape(T, D), x,
                                      np.asarray(scale).reshape(rows, D))
    dx = np.empty((T, D), dtype=np.float64)
    dshift = np.empty((rows, D), dtype=np.float64)
    dscale = np.empty((rows, D), dtype=np.float64)
    rc = (lib or load()).lnmod_oracle_backward(_ptr(dy_c), _ptr(x_c), _ptr(sc_c), f32, _ptr(cu),
                                               nseg, D, float(eps), int(mod),
                                               _ptr(dx), _ptr(dshift), _ptr(dscale))
    if rc != 0:
        raise RuntimeError("lnmod_oracle_backward failed with status %d" % rc)
    return dx, dshift, dscale
