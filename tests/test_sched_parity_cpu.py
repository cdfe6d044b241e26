"""Parity of the library's host-side scheduling entry points (include/lnmod_sched.h, paper
Sec. 3.2) with the plain reference in oracle/sched_oracle.py, through the C ABI.  No GPU is
needed: the functions never touch a device.  Integer results must match exactly (both sides take
floor(M/S^p) in double with the C library's pow); fitted parameters to 1e-9 relative."""
import math
import os
import re

import numpy as np
import pytest

from oracle import sched_oracle as so
from paper_2605_17923_amd import lnmod, sched

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _lib():
    if not os.path.exists(lnmod.LIBRARY):
        from paper_2605_17923_amd.build import build_library
        build_library()
    return lnmod.library()


def test_header_symbols_are_exported_and_bound(_lib):
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "lnmod_sched.h")).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(lnmod_[a-z_0-9]+)\s*\(", text)))
    assert set(names) == set(sched.EXPORTS)
    for n in names:
        assert hasattr(_lib, n) and callable(getattr(sched, n))


def test_eq2_matches_reference_exactly():
    rng = np.random.default_rng(11)
    lengths = [1, 2, 77, 256, 1560, 4096, 8190, 16380, 20000, 32760, 75600, 152880, 10 ** 6]
    lengths += [int(v) for v in rng.integers(1, 200000, 300)]
    for M_mem, M_comp, p in ((262144.0, 2.0e9, 2.0), (131072.0, 3.7e8, 1.85), (1e6, 5e10, 2.37), (5e5, 1e300, 2.0),
                             (0.0, 0.0, 2.0), (3e5, 1e7, 1.6), (1.5e5, 8.8e9, 2.4)):
        rc, got = sched.lnmod_bucket_batch_sizes(lengths, M_mem, M_comp, p)
        assert rc == 0
        want = [so.bucket_batch_size(S, M_mem, M_comp, p) for S in lengths]
        assert got == want
        assert all(sched.lnmod_bucket_batch_size(S, M_mem, M_comp, p) == w for S, w in zip(lengths[:20], want))
    # the paper's point: long buckets are cut below the equal-token batch, short ones are not
    eq_token = [max(1, math.floor(262144.0 / S)) for S in (1024, 32760)]
    assert sched.lnmod_bucket_batch_size(1024, 262144.0, 2.0e9, 2.0) == eq_token[0]
    assert sched.lnmod_bucket_batch_size(32760, 262144.0, 2.0e9, 2.0) < eq_token[1]


def test_eq2_rejects_bad_arguments():
    f = sched.lnmod_bucket_batch_size
    assert f(0, 1e5, 1e9, 2.0) == 0 and f(-5, 1e5, 1e9, 2.0) == 0
    assert f(10, float("nan"), 1e9, 2.0) == 0 and f(10, 1e5, float("inf"), 2.0) == 0
    assert f(10, -1.0, 1e9, 2.0) == 0 and f(10, 1e5, 1e9, float("nan")) == 0
    assert sched.lnmod_bucket_batch_sizes([], 1e5, 1e9, 2.0) == (0, [])


def _measurements(a, b, p, noise, seed):
    rng = np.random.default_rng(seed)
    S = rng.choice([1560, 4096, 8190, 16380, 20000, 24000, 32760, 50000, 75600], size=40)
    B = rng.integers(1, 9, size=40)
    t = (a + b * B * S.astype(np.float64) ** p) * (1.0 + noise * rng.standard_normal(40))
    return B, S, t


@pytest.mark.parametrize("a,b,p,noise,seed", [(0.35, 2.5e-10, 2.0, 0.0, 1), (1.2, 4e-9, 1.73, 0.0, 2),
                                              (0.5, 3e-10, 1.9, 0.01, 3), (0.1, 1e-11, 2.4, 0.03, 4),
                                              (0.8, 3e-8, 1.6, 0.05, 5), (0.0, 1e-9, 2.2, 0.2, 6)])
def test_fit_matches_reference(a, b, p, noise, seed):
    B, S, t = _measurements(a, b, p, noise, seed)
    for step in (0.01, 0.05, 0.2):
        rc, fa, fb, fp, r2 = sched.lnmod_fit_cost_model(B, S, t, 1.6, 2.4, step)
        wa, wb, wp, wr2 = so.fit_cost_model(B, S, t, 1.6, 2.4, step)
        assert rc == 0
        assert fp == pytest.approx(wp, abs=1e-12)
        assert r2 == pytest.approx(wr2, rel=1e-9, abs=1e-12)
        assert fb == pytest.approx(wb, rel=1e-8) and fa == pytest.approx(wa, rel=1e-7, abs=1e-9 * abs(t).max())
        assert sched.lnmod_comp_bound(2.0 * t.mean(), fa, fb) == pytest.approx(so.comp_bound(2.0 * t.mean(), wa, wb), rel=1e-7)


def test_fit_rejects_bad_arguments_and_degenerate_data():
    B, S, t = _measurements(0.3, 1e-10, 2.0, 0.0, 9)
    f = sched.lnmod_fit_cost_model
    assert f(B[:1], S[:1], t[:1])[0] == 1
    assert f(B, S, t, 1.6, 2.4, 0.0)[0] == 1 and f(B, S, t, 2.4, 1.6, 0.01)[0] == 1
    bad = t.copy()
    bad[3] = float("nan")
    assert f(B, S, bad)[0] == 1
    zero_b = B.copy()
    zero_b[0] = 0
    assert f(zero_b, S, t)[0] == 1
    assert f(B, S, np.full(t.size, 3.0))[0] == 2                          # all step times equal
    assert f(np.full(5, 2), np.full(5, 1000), np.arange(5.0))[0] == 2     # all z equal
    assert sched.lnmod_comp_bound(1.0, 2.0, 1e-9) == 0.0 and sched.lnmod_comp_bound(1.0, 0.1, 0.0) == 0.0
