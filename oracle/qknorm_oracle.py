"""ctypes front end of the float64 CPU oracle of the fused Q-Norm + K-Norm operator
(qknorm_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  The product package never imports this module, and this module imports
nothing from the product package.  The arithmetic lives entirely in qknorm_oracle.c (its header
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
SOURCE = os.path.join(_HERE, "qknorm_oracle.c")
LIBRARY = os.path.join(_HERE, "libqknorm_oracle.so")

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
        lib.qknorm_oracle_forward.restype = cint
        lib.qknorm_oracle_forward.argtypes = [vp, vp, cint, i64, i64, dbl, vp, vp]
        lib.qknorm_oracle_backward.restype = cint
        lib.qknorm_oracle_backward.argtypes = [vp, vp, vp, cint, i64, i64, dbl, vp, vp]
        if path is None:
            _lib = lib
        return lib


def _carrier(*arrays):
    f32 = all(np.asarray(a).dtype == np.float32 for a in arrays)
    dt = np.float32 if f32 else np.float64
    return [np.ascontiguousarray(a, dtype=dt) for a in arrays], int(f32)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def forward_one(x, w, eps=1e-6, lib=None):
    """y [N, D], rstd [N] of one tensor in float64."""
    x = np.asarray(x)
    N, D = x.shape
    (x_c, w_c), f32 = _carrier(x, np.asarray(w).reshape(D))
    y = np.empty((N, D), dtype=np.float64)
    rstd = np.empty(N, dtype=np.float64)
    rc = (lib or load()).qknorm_oracle_forward(_ptr(x_c), _ptr(w_c), f32, N, D, float(eps),
                                               _ptr(y), _ptr(rstd))
    if rc != 0:
        raise RuntimeError("qknorm_oracle_forward failed with status %d" % rc)
    return y, rstd


def backward_one(dy, x, w, eps=1e-6, lib=None):
    """dx [N, D], dw [D] of one tensor in float64 (rstd recomputed from x)."""
    x = np.asarray(x)
    N, D = x.shape
    (dy_c, x_c, w_c), f32 = _carrier(np.asarray(dy).reshape(N, D), x, np.asarray(w).reshape(D))
    dx = np.empty((N, D), dtype=np.float64)
    dw = np.empty(D, dtype=np.float64)
    rc = (lib or load()).qknorm_oracle_backward(_ptr(dy_c), _ptr(x_c), _ptr(w_c), f32, N, D,
                                                float(eps), _ptr(dx), _ptr(dw))
    if rc != 0:
        raise RuntimeError("qknorm_oracle_backward failed with status %d" % rc)
    return dx, dw


def forward(q, k, wq, wk, eps=1e-6, lib=None):
    """-> q_out, k_out, rstd_q, rstd_k: the operator is the same normalisation on both tensors."""
    yq, rq = forward_one(q, wq, eps, lib)
    yk, rk = forward_one(k, wk, eps, lib)
    return yq, yk, rq, rk


def backward(dq_out, dk_out, q, k, wq, wk, eps=1e-6, lib=None):
    """-> dq, dk, dwq, dwk."""
    dq, dwq = backward_one(dq_out, q, wq, eps, lib)
    dk, dwk = backward_one(dk_out, k, wk, eps, lib)
    return dq, dk, dwq, dwk
