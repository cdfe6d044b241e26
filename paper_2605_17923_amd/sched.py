"""Thin Python binding of the host-side scheduling entry points of liblnmod.so (the C ABI in
include/lnmod_sched.h): Eq. 2's bucket batch size and the cost-model fit of the paper's Sec. 3.2.
Argument marshalling only; there is no Python fallback: without the built library every call
raises."""
from __future__ import annotations

import ctypes

from . import lnmod as _lnmod

EXPORTS = ("lnmod_bucket_batch_size", "lnmod_bucket_batch_sizes", "lnmod_fit_cost_model",
           "lnmod_comp_bound")

_ready = False


def _lib():
    global _ready
    lib = _lnmod.library()
    if not _ready:
        i64, dbl, cint = ctypes.c_int64, ctypes.c_double, ctypes.c_int
        pi64, pdbl = ctypes.POINTER(i64), ctypes.POINTER(dbl)
        lib.lnmod_bucket_batch_size.restype = i64
        lib.lnmod_bucket_batch_size.argtypes = [i64, dbl, dbl, dbl]
        lib.lnmod_bucket_batch_sizes.restype = cint
        lib.lnmod_bucket_batch_sizes.argtypes = [pi64, i64, dbl, dbl, dbl, pi64]
        lib.lnmod_fit_cost_model.restype = cint
        lib.lnmod_fit_cost_model.argtypes = [pi64, pi64, pdbl, i64, dbl, dbl, dbl, pdbl, pdbl, pdbl, pdbl]
        lib.lnmod_comp_bound.restype = dbl
        lib.lnmod_comp_bound.argtypes = [dbl, dbl, dbl]
        _ready = True
    return lib


def lnmod_bucket_batch_size(S, M_mem, M_comp, p):
    return int(_lib().lnmod_bucket_batch_size(int(S), float(M_mem), float(M_comp), float(p)))


def lnmod_bucket_batch_sizes(S, M_mem, M_comp, p):
    """-> (status, list of batch sizes) for a sequence of bucket lengths."""
    n = len(S)
    arr = (ctypes.c_int64 * max(n, 1))(*[int(v) for v in S])
    out = (ctypes.c_int64 * max(n, 1))()
    rc = _lib().lnmod_bucket_batch_sizes(arr, n, float(M_mem), float(M_comp), float(p), out)
    return int(rc), [int(out[i]) for i in range(n)]


def lnmod_fit_cost_model(B, S, step_time, p_lo=1.6, p_hi=2.4, p_step=0.01):
    """-> (status, a, b, p, r2)."""
    n = len(B)
    Ba = (ctypes.c_int64 * max(n, 1))(*[int(v) for v in B])
    Sa = (ctypes.c_int64 * max(n, 1))(*[int(v) for v in S])
    ta = (ctypes.c_double * max(n, 1))(*[float(v) for v in step_time])
    a, b, p, r2 = (ctypes.c_double() for _ in range(4))
    rc = _lib().lnmod_fit_cost_model(Ba, Sa, ta, n, float(p_lo), float(p_hi), float(p_step),
                                     ctypes.byref(a), ctypes.byref(b), ctypes.byref(p), ctypes.byref(r2))
    return int(rc), a.value, b.value, p.value, r2.value


def lnmod_comp_bound(target_sync, a, b):
    return float(_lib().lnmod_comp_bound(float(target_sync), float(a), float(b)))
