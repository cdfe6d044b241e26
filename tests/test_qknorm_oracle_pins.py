"""Pins for the float64 oracle of the fused Q-Norm + K-Norm operator (oracle/qknorm_oracle.c):
exact-rational brute force, closed forms, invariants the mathematics fixes, torch's float64
rms_norm + autograd (a library routine) and finite differences; then planted mistakes in a copy
of the C source, each of which a pin has to notice.

The paper only names this fusion (Sec. 4.4); the definition is the query/key RMS normalisation
with a learned weight of MMDiT-style attention blocks."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import qknorm_oracle as qo

PIN_FUNCS = []


def pin(f):
    PIN_FUNCS.append(f)
    return f


def _rng(seed):
    return np.random.default_rng(seed)


@pin
def test_bruteforce_tiny(lib=None):
    rng = _rng(1)
    N, D, eps = 3, 5, 1e-3
    x, w, dy = rng.normal(0.4, 1.3, (N, D)), rng.normal(1, 0.3, D), rng.normal(0, 1, (N, D))
    y, r = qo.forward_one(x, w, eps, lib)
    dx, dw = qo.backward_one(dy, x, w, eps, lib)
    F = Fraction
    edw = [0.0] * D
    for n in range(N):
        row = [F(float(v)) for v in x[n]]
        ms = sum(v * v for v in row) / D
        rr = 1.0 / math.sqrt(float(ms + F(eps)))
        assert r[n] == pytest.approx(rr, rel=1e-13)
        xhat = [float(v) * rr for v in row]
        g = [float(dy[n, d]) * float(w[d]) for d in range(D)]
        c = sum(g[d] * xhat[d] for d in range(D)) / D
        for d in range(D):
            assert y[n, d] == pytest.approx(xhat[d] * w[d], rel=1e-12, abs=1e-14)
            assert dx[n, d] == pytest.approx(rr * (g[d] - xhat[d] * c), rel=1e-10, abs=1e-12)
            edw[d] += float(dy[n, d]) * xhat[d]
    for d in range(D):
        assert dw[d] == pytest.approx(edw[d], rel=1e-11, abs=1e-12)


@pin
def test_closed_forms(lib=None):
    # constant-magnitude row (+a, -a, ...): ms = a^2, xhat = +-a/sqrt(a^2+eps)
    a, eps, D = 3.0, 7.0, 6                       # a^2 + eps = 16
    x = np.array([[a, -a, a, -a, a, -a]])
    w = np.arange(1.0, D + 1)
    y, r = qo.forward_one(x, w, eps, lib)
    assert r[0] == pytest.approx(0.25, rel=1e-15)
    assert np.allclose(y[0], x[0] * 0.25 * w, rtol=1e-15)
    # single non-zero entry: ms = v^2/D
    x = np.zeros((1, 4))
    x[0, 2] = 6.0
    y, r = qo.forward_one(x, np.ones(4), 0.0 + 7.0, lib)       # 36/4 + 7 = 16
    assert r[0] == pytest.approx(0.25, rel=1e-15) and y[0].tolist() == [0.0, 0.0, 1.5, 0.0]
    # zero row: r = 1/sqrt(eps), y = 0, dx = r * g
    dy = np.array([[1.0, -2.0, 0.5, 4.0]])
    y, r = qo.forward_one(np.zeros((1, 4)), np.ones(4) * 2, 1e-4, lib)
    dx, dw = qo.backward_one(dy, np.zeros((1, 4)), np.ones(4) * 2, 1e-4, lib)
    assert r[0] == pytest.approx(100.0, rel=1e-14) and np.all(y == 0)
    assert np.allclose(dx, 100.0 * 2 * dy, rtol=1e-14) and np.all(dw == 0)


@pin
def test_invariants(lib=None):
    rng = _rng(2)
    N, D, eps = 9, 48, 1e-2
    x, w, dy = rng.normal(0.2, 1.1, (N, D)), rng.normal(1, 0.2, D), rng.normal(0, 1, (N, D))
    one = np.ones(D)
    y, r = qo.forward_one(x, one, eps, lib)
    ms = (x ** 2).mean(axis=1)
    assert np.allclose((y ** 2).mean(axis=1), ms / (ms + eps), rtol=1e-13)       # mean square of xhat
    # scale covariance: RMS(alpha x; eps alpha^2) = sign(alpha) RMS(x; eps); no shift invariance
    for alpha in (-3.0, 0.25):
        y2, r2 = qo.forward_one(alpha * x, one, eps * alpha * alpha, lib)
        assert np.allclose(y2, np.sign(alpha) * y, rtol=1e-12, atol=1e-14)
        assert np.allclose(r2, r / abs(alpha), rtol=1e-13)
    assert not np.allclose(qo.forward_one(x + 1.0, one, eps, lib)[0], y, atol=1e-3)
    # the weight is a plain per-feature factor
    yw, _ = qo.forward_one(x, w, eps, lib)
    assert np.allclose(yw, y * w, rtol=1e-14, atol=0)
    # backward: sum_d dx*x = r*D*c*eps/(ms+eps) per row; dw independent of w; dx linear in dy
    dx, dw = qo.backward_one(dy, x, w, eps, lib)
    xhat = x * r[:, None]
    c = ((dy * w) * xhat).mean(axis=1)
    assert np.allclose((dx * x).sum(axis=1), D * c * eps / (ms + eps), rtol=1e-9, atol=1e-12)
    assert np.allclose(dw, (dy * xhat).sum(axis=0), rtol=1e-12, atol=1e-13)
    dx2, dw2 = qo.backward_one(2 * dy, x, 3 * w, eps, lib)
    assert np.allclose(dx2, 6 * dx, rtol=1e-12, atol=1e-14) and np.allclose(dw2, 2 * dw, rtol=1e-12, atol=1e-14)


@pin
def test_against_torch_rms_norm_autograd(lib=None):
    rng = _rng(3)
    N, D, eps = 11, 40, 1e-5
    x, w, dy = rng.normal(0, 1.5, (N, D)), rng.normal(1, 0.3, D), rng.normal(0, 1, (N, D))
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    yt = torch.nn.functional.rms_norm(xt, (D,), wt, eps)
    (torch.tensor(dy) * yt).sum().backward()
    y, r = qo.forward_one(x, w, eps, lib)
    dx, dw = qo.backward_one(dy, x, w, eps, lib)
    assert np.allclose(y, yt.detach().numpy(), rtol=1e-12, atol=1e-14)
    assert np.allclose(dx, xt.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(dw, wt.grad.numpy(), rtol=1e-11, atol=1e-12)


@pin
def test_finite_differences(lib=None):
    rng = _rng(4)
    N, D, eps = 4, 10, 1e-3
    x, w, dy = rng.normal(0, 1, (N, D)), rng.normal(1, 0.3, D), rng.normal(0, 1, (N, D))
    dx, dw = qo.backward_one(dy, x, w, eps, lib)

    def loss(xx, ww):
        return float((dy * qo.forward_one(xx, ww, eps, lib)[0]).sum())

    step = 1e-6
    for _ in range(12):
        n, d = int(rng.integers(0, N)), int(rng.integers(0, D))
        xp, xm = x.copy(), x.copy()
        xp[n, d] += step
        xm[n, d] -= step
        assert (loss(xp, w) - loss(xm, w)) / (2 * step) == pytest.approx(dx[n, d], rel=2e-6, abs=2e-8)
        wp, wm = w.copy(), w.copy()
        wp[d] += step
        wm[d] -= step
        assert (loss(x, wp) - loss(x, wm)) / (2 * step) == pytest.approx(dw[d], rel=2e-6, abs=2e-8)


@pin
def test_pair_is_two_independent_halves(lib=None):
    rng = _rng(5)
    N, D = 6, 16
    q, k = rng.normal(0, 1, (N, D)).astype(np.float32), rng.normal(0, 2, (N, D)).astype(np.float32)
    wq, wk = rng.normal(1, 0.1, D).astype(np.float32), rng.normal(1, 0.1, D).astype(np.float32)
    dq, dk = rng.normal(0, 1, (N, D)).astype(np.float32), rng.normal(0, 1, (N, D)).astype(np.float32)
    yq, yk, rq, rk = qo.forward(q, k, wq, wk, lib=lib)
    assert np.array_equal(yq, qo.forward_one(q, wq, lib=lib)[0]) and np.array_equal(yk, qo.forward_one(k, wk, lib=lib)[0])
    a, b, c, d = qo.backward(dq, dk, q, k, wq, wk, lib=lib)
    assert np.array_equal(a, qo.backward_one(dq, q, wq, lib=lib)[0]) and np.array_equal(d, qo.backward_one(dk, k, wk, lib=lib)[1])
    # float32 carriers give the same numbers as the same values passed as float64
    assert np.array_equal(yq, qo.forward_one(q.astype(np.float64), wq.astype(np.float64), lib=lib)[0])
    # empty input
    y0, r0 = qo.forward_one(np.zeros((0, D)), wq, lib=lib)
    dx0, dw0 = qo.backward_one(np.zeros((0, D)), np.zeros((0, D)), wq, lib=lib)
    assert y0.shape == (0, D) and r0.shape == (0,) and np.all(dw0 == 0)


MUTANTS = [
    ("mean of squares divides by D-1", "const double r = 1.0 / sqrt(s / (double)D + eps);",
     "const double r = 1.0 / sqrt(s / (double)(D - 1) + eps);", 0),
    ("eps outside the sqrt", "const double r = 1.0 / sqrt(s / (double)D + eps);",
     "const double r = 1.0 / (sqrt(s / (double)D) + eps);", 0),
    ("eps dropped", "const double r = 1.0 / sqrt(s / (double)D + eps);", "const double r = 1.0 / sqrt(s / (double)D);", 0),
    ("sum of x instead of x^2", "s += v * v;", "s += v;", 0),
    ("centred like a LayerNorm", "y[n * D + d] = (ld(x, in_f32, n * D + d) * r) * ld(w, in_f32, d);",
     "y[n * D + d] = ((ld(x, in_f32, n * D + d) - s / (double)D) * r) * ld(w, in_f32, d);", 0),
    ("weight as 1+w", "* r) * ld(w, in_f32, d);", "* r) * (1.0 + ld(w, in_f32, d));", 0),
    ("weight dropped", "* r) * ld(w, in_f32, d);", "* r);", 0),
    ("rstd saved as rms", "rstd[n] = r;", "rstd[n] = 1.0 / r;", 0),
    ("backward: eps dropped", "r[n] = 1.0 / sqrt(s / (double)D + eps);", "r[n] = 1.0 / sqrt(s / (double)D);", 0),
    ("backward: g without the weight", "const double g = ld(dy, in_f32, n * D + d) * ld(w, in_f32, d);",
     "const double g = ld(dy, in_f32, n * D + d);", 1),
    ("backward: c without the weight", "const double g = ld(dy, in_f32, n * D + d) * ld(w, in_f32, d);",
     "const double g = ld(dy, in_f32, n * D + d);", 0),
    ("backward: projection term dropped", "dx[n * D + d] = r[n] * (g - xhat * c);", "dx[n * D + d] = r[n] * g;", 0),
    ("backward: projection term sign", "dx[n * D + d] = r[n] * (g - xhat * c);", "dx[n * D + d] = r[n] * (g + xhat * c);", 0),
    ("backward: a LayerNorm's mean term", "dx[n * D + d] = r[n] * (g - xhat * c);",
     "dx[n * D + d] = r[n] * (g - sc * 0.0 - xhat * c) - r[n] * ld(dy, in_f32, n * D) / (double)D;", 0),
    ("backward: dx not scaled by rstd", "dx[n * D + d] = r[n] * (g - xhat * c);", "dx[n * D + d] = (g - xhat * c);", 0),
    ("dw sums dy only", "dw[d] += ld(dy, in_f32, n * D + d) * (ld(x, in_f32, n * D + d) * r[n]);", "dw[d] += ld(dy, in_f32, n * D + d);", 0),
    ("dw uses x without rstd", "dw[d] += ld(dy, in_f32, n * D + d) * (ld(x, in_f32, n * D + d) * r[n]);",
     "dw[d] += ld(dy, in_f32, n * D + d) * ld(x, in_f32, n * D + d);", 0),
    ("dw skips the last row", "for (int64_t n = 0; n < N; ++n)\n            for (int64_t d = d0; d < d1; ++d)",
     "for (int64_t n = 0; n < N - 1; ++n)\n            for (int64_t d = d0; d < d1; ++d)", 0),
]


def _replace_nth(text, old, new, nth):
    pos = -1
    for _ in range(nth + 1):
        pos = text.find(old, pos + 1)
        if pos < 0:
            raise AssertionError("mutation site not found: %r (occurrence %d)" % (old, nth))
    return text[:pos] + new + text[pos + len(old):]


@pytest.mark.parametrize("label,old,new,nth", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_mutant(tmp_path, label, old, new, nth):
    with open(qo.SOURCE) as f:
        src = f.read()
    mutated = _replace_nth(src, old, new, nth)
    assert mutated != src
    c_path = os.path.join(tmp_path, "mutant.c")
    with open(c_path, "w") as f:
        f.write(mutated)
    lib = qo.load(qo.build(force=True, source=c_path, output=os.path.join(tmp_path, "libmutant.so")))
    caught = []
    for check in PIN_FUNCS:
        try:
            check(lib)
        except AssertionError:
            caught.append(check.__name__)
    assert caught, "no pin notices the planted mistake: " + label


def test_unmutated_source_passes_every_pin(tmp_path):
    lib = qo.load(qo.build(force=True, source=qo.SOURCE, output=os.path.join(tmp_path, "libclean.so")))
    for check in PIN_FUNCS:
        check(lib)
