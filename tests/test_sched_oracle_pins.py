"""Pins for the plain reference of the dual-constraint bucket sizing and its cost-model fit
(oracle/sched_oracle.py, paper Sec. 3.2, Eq. 2): exact integer brute force, the special cases the
text describes (memory-bound short buckets, compute-bound long buckets, the equal-token scheme as
the limit of a huge compute bound, never below one), planted parameters recovered by the fit,
scipy's linregress as a library cross-check, and invariances of R^2.  The last test plants
mistakes in a copy of the reference's source and requires a pin to notice each."""
import math
from fractions import Fraction

import numpy as np
import pytest
from scipy import stats

from oracle import sched_oracle as so

PIN_FUNCS = []


def pin(f):
    PIN_FUNCS.append(f)
    return f


@pin
def test_eq2_bruteforce_integer_exponent(mod=so):
    # p = 2 and integer bounds: B is the largest integer with B*S <= M_mem and B*S^2 <= M_comp, at least 1
    for S in (1, 7, 256, 1560, 8190, 32760, 75600):
        for M_mem, M_comp in ((131072, 10 ** 9), (300000, 4 * 10 ** 9), (10, 10), (75600, 75600 ** 2), (0, 0)):
            want = 0
            while (want + 1) * S <= M_mem and (want + 1) * S * S <= M_comp:
                want += 1
            want = max(1, want)
            assert mod.bucket_batch_size(S, float(M_mem), float(M_comp), 2.0) == want, (S, M_mem, M_comp)
            # the same through exact rationals
            f = max(1, min(Fraction(M_mem, S).__floor__(), Fraction(M_comp, S * S).__floor__()))
            assert f == want


@pin
def test_eq2_regimes(mod=so):
    M_mem, M_comp, p = 262144.0, 2.0e9, 2.0
    cross = (M_comp / M_mem) ** (1.0 / (p - 1.0))            # S where both bounds meet: 7629.4
    assert mod.bucket_batch_size(1024, M_mem, M_comp, p) == 256                 # memory-bound: M_mem / S
    assert mod.bucket_batch_size(int(cross) - 100, M_mem, M_comp, p) == math.floor(M_mem / (int(cross) - 100))
    assert mod.bucket_batch_size(int(cross) + 100, M_mem, M_comp, p) == math.floor(M_comp / (int(cross) + 100) ** 2)
    assert mod.bucket_batch_size(32760, M_mem, M_comp, p) == 1                  # 2e9 / 32760^2 = 1.86
    assert mod.bucket_batch_size(75600, M_mem, M_comp, p) == 1                  # never below one
    # a huge compute bound gives the equal-token scheme B*S ~ constant
    for S in (100, 999, 40000):
        assert mod.bucket_batch_size(S, M_mem, 1e300, p) == max(1, math.floor(M_mem / S))
    # a larger exponent can only shrink the batch; non-integer exponents go through pow
    assert mod.bucket_batch_size(5000, M_mem, M_comp, 2.2) <= mod.bucket_batch_size(5000, M_mem, M_comp, 1.8)
    assert mod.bucket_batch_size(5000, 1e9, M_comp, 1.85) == math.floor(M_comp / 5000 ** 1.85)


def _measurements(a, b, p, noise=0.0, seed=0):
    rng = np.random.default_rng(seed)
    S = np.array([1560, 4096, 8190, 16380, 20000, 24000, 32760, 32760, 50000, 75600, 75600, 2048])
    B = np.array([16, 8, 4, 2, 1, 2, 1, 2, 1, 1, 2, 32])
    t = a + b * B * S.astype(np.float64) ** p
    if noise:
        t = t * (1.0 + noise * rng.standard_normal(t.size))
    return B, S, t


@pin
def test_fit_recovers_planted_parameters(mod=so):
    for a, b, p in ((0.35, 2.5e-10, 2.0), (1.2, 4.0e-9, 1.73), (0.0, 1e-11, 2.4), (0.8, 3e-8, 1.6)):
        B, S, t = _measurements(a, b, p)
        fa, fb, fp, r2 = mod.fit_cost_model(B, S, t, 1.6, 2.4, 0.01)
        assert fp == pytest.approx(p, abs=1e-9) and r2 == pytest.approx(1.0, abs=1e-9)
        assert fa == pytest.approx(a, rel=1e-6, abs=1e-6) and fb == pytest.approx(b, rel=1e-6)
    # with 0.2 % noise the exponent lands within a few grid steps and R^2 stays high
    B, S, t = _measurements(0.5, 3e-10, 1.9, noise=0.002, seed=3)
    fa, fb, fp, r2 = mod.fit_cost_model(B, S, t, 1.6, 2.4, 0.01)
    assert abs(fp - 1.9) <= 0.04 and r2 > 0.9999
    # the grid is honoured: a coarse grid can only return its own points, end points included
    fa, fb, fp, r2 = mod.fit_cost_model(B, S, t, 1.6, 2.4, 0.2)
    assert min(abs(fp - g) for g in (1.6, 1.8, 2.0, 2.2, 2.4)) < 1e-9
    assert mod.fit_cost_model(*_measurements(0.1, 1e-11, 2.4), 1.6, 2.4, 0.1)[2] == pytest.approx(2.4, abs=1e-9)
    assert mod.p_grid(1.6, 2.4, 0.01)[-1] == pytest.approx(2.4, abs=1e-9) and len(mod.p_grid(1.6, 2.4, 0.01)) == 81


@pin
def test_fit_against_linregress_and_invariances(mod=so):
    B, S, t = _measurements(0.4, 2e-10, 2.1, noise=0.05, seed=7)
    for p in (1.6, 2.0, 2.37):
        a, b, r2 = mod.fit_at(B, S, t, p)
        lr = stats.linregress(B * S.astype(np.float64) ** p, t)
        assert a == pytest.approx(lr.intercept, rel=1e-8, abs=1e-10)
        assert b == pytest.approx(lr.slope, rel=1e-8)
        assert r2 == pytest.approx(lr.rvalue ** 2, rel=1e-8)
    # R^2 and the chosen p do not change under an affine change of the time unit
    f1 = mod.fit_cost_model(B, S, t, 1.6, 2.4, 0.01)
    f2 = mod.fit_cost_model(B, S, 1000.0 * t + 5.0, 1.6, 2.4, 0.01)
    assert f1[2] == f2[2] and f1[3] == pytest.approx(f2[3], rel=1e-9)
    assert f2[1] == pytest.approx(1000.0 * f1[1], rel=1e-7) and f2[0] == pytest.approx(1000.0 * f1[0] + 5.0, rel=1e-7)
    # the order of the measurements does not matter
    perm = np.random.default_rng(1).permutation(t.size)
    f3 = mod.fit_cost_model(B[perm], S[perm], t[perm], 1.6, 2.4, 0.01)
    assert f3[2] == f1[2] and f3[3] == pytest.approx(f1[3], rel=1e-9)


@pin
def test_comp_bound_closes_the_loop(mod=so):
    a, b, p, target = 0.35, 2.5e-10, 2.0, 6.0
    m = mod.comp_bound(target, a, b)
    assert m == pytest.approx((target - a) / b, rel=1e-15)
    # a bucket sized by that bound meets the target, one more sample would not
    for S in (20000, 32760, 50000):
        Bs = mod.bucket_batch_size(S, 1e12, m, p)
        assert a + b * Bs * S ** p <= target * (1 + 1e-12)
        assert Bs == 1 or a + b * (Bs + 1) * S ** p > target
    assert mod.comp_bound(0.2, a, b) == 0.0 and mod.comp_bound(target, a, 0.0) == 0.0
    assert mod.comp_bound(target, a, -1.0) == 0.0


MUTANTS = [
    ("ceil instead of floor (memory)", "by_mem = math.floor(M_mem / S)", "by_mem = math.ceil(M_mem / S)"),
    ("ceil instead of floor (compute)", "by_comp = math.floor(M_comp / math.pow(S, p))", "by_comp = math.ceil(M_comp / math.pow(S, p))"),
    ("max of the two bounds", "return max(1, min(by_mem, by_comp))", "return max(1, max(by_mem, by_comp))"),
    ("no lower bound of one", "return max(1, min(by_mem, by_comp))", "return min(by_mem, by_comp)"),
    ("compute bound linear in S", "math.pow(S, p))", "S)"),
    ("compute bound multiplied", "by_comp = math.floor(M_comp / math.pow(S, p))", "by_comp = math.floor(M_comp * math.pow(S, p))"),
    ("grid misses its end point", "return [p_lo + g * p_step for g in range(steps + 1)]", "return [p_lo + g * p_step for g in range(steps)]"),
    ("model without B", "z = B * np.power(S, p)", "z = np.power(S, p)"),
    ("model without the intercept", "A = np.stack([np.ones_like(z), z], axis=1)", "A = np.stack([np.zeros_like(z), z], axis=1)"),
    ("keeps the smallest R^2", "if best is None or r[2] > best[3]:", "if best is None or r[2] < best[3]:"),
    ("R^2 as SSE/SST", "return float(a), float(b), 1.0 - sse / sst", "return float(a), float(b), sse / sst"),
    ("comp bound forgets the intercept", "m = (target_sync - a) / b", "m = target_sync / b"),
    ("comp bound multiplies", "m = (target_sync - a) / b", "m = (target_sync - a) * b"),
]


@pytest.mark.parametrize("label,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_mutant(label, old, new):
    import types
    src = open(so.__file__).read()
    assert src.count(old) == 1, "mutation site not unique: " + old
    mod = types.ModuleType("sched_mutant")
    exec(compile(src.replace(old, new), "sched_mutant", "exec"), mod.__dict__)
    caught = []
    for check in PIN_FUNCS:
        try:
            check(mod)
        except (AssertionError, ValueError, ZeroDivisionError, OverflowError, IndexError, TypeError):
            caught.append(check.__name__)
    assert caught, "no pin notices the planted mistake: " + label
