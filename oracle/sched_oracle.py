"""Plain reference of the dual-constraint bucket sizing and its cost-model fit (paper Sec. 3.2).

TEST INFRASTRUCTURE ONLY: imported by tests/ and by nothing in the product package.  Slow and
literal on purpose; it shares no code with the C++ implementation.

Eq. 2:   B_shape = max(1, min(floor(M_mem / S), floor(M_comp / S^p)))

Fit:     step_time ~ a + b * B * S^p; for every p on the grid p_lo, p_lo + p_step, ..., p_hi the
         ordinary least-squares line of step_time on z = B * S^p (numpy.linalg.lstsq, a library
         routine) and its coefficient of determination R^2 = 1 - SSE/SST; the first grid point
         with the largest R^2 is kept.  Then M_comp = (target_sync - a) / b.
"""
from __future__ import annotations

import math

import numpy as np


def bucket_batch_size(S: int, M_mem: float, M_comp: float, p: float) -> int:
    by_mem = math.floor(M_mem / S)
    by_comp = math.floor(M_comp / math.pow(S, p))
    return max(1, min(by_mem, by_comp))


def p_grid(p_lo: float, p_hi: float, p_step: float):
    steps = int(math.floor((p_hi - p_lo) / p_step + 1e-9))
    return [p_lo + g * p_step for g in range(steps + 1)]


def fit_at(B, S, t, p: float):
    """(a, b, R^2) of the least-squares line of t on z = B * S^p, or None if z is constant."""
    B = np.asarray(B, dtype=np.float64)
    S = np.asarray(S, dtype=np.float64)
    t = np.asarray(t, dtype=np.float64)
    z = B * np.power(S, p)
    if np.all(z == z[0]):
        return None
    A = np.stack([np.ones_like(z), z], axis=1)
    (a, b), *_ = np.linalg.lstsq(A, t, rcond=None)
    sse = float(np.sum((t - (a + b * z)) ** 2))
    sst = float(np.sum((t - t.mean()) ** 2))
    return float(a), float(b), 1.0 - sse / sst


def fit_cost_model(B, S, t, p_lo: float = 1.6, p_hi: float = 2.4, p_step: float = 0.01):
    """-> (a, b, p, R^2) of the best grid point."""
    best = None
    for p in p_grid(p_lo, p_hi, p_step):
        r = fit_at(B, S, t, p)
        if r is None:
            continue
        if best is None or r[2] > best[3]:
            best = (r[0], r[1], p, r[2])
    if best is None:
        raise ValueError("degenerate fit")
    return best


def comp_bound(target_sync: float, a: float, b: float) -> float:
    if not b > 0.0:
        return 0.0
    m = (target_sync - a) / b
    return m if (math.isfinite(m) and m > 0.0) else 0.0
