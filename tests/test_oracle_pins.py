"""Pins for the float64 CPU oracle: everything here checks oracle/ against something that is
not the oracle -- exact rational brute force, closed forms, invariants the mathematics fixes,
a library routine (torch layer_norm + autograd in float64) and finite differences.

The operator is the fused LayerNorm-Modulate of the paper's Sec. 3.3 (LayerNorm without
affine, biased variance, eps inside the square root, then y = xhat*(1+scale)+shift; the
backward gives dx and the modulation gradients summed along the token axis).  The paper prints
no worked numeric example of it, so there is no published value to pin to; tests/golden holds
one hand-derived closed-form case instead.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

PIN_FUNCS = []          # (name, callable(lib)) used again by the mutation test


def pin(f):
    PIN_FUNCS.append(f)
    return f


def _rng(seed):
    return np.random.default_rng(seed)


# --------------------------------------------------------------------------------------------
# 1. exact rational brute force on tiny inputs (literal per-element loops, no numpy math)
# --------------------------------------------------------------------------------------------
def _bf_forward(x, shift, scale, seg_of, eps):
    """Literal definition with Fractions; the only float step is the square root."""
    T, D = len(x), len(x[0])
    y = [[0.0] * D for _ in range(T)]
    mean, rstd = [0.0] * T, [0.0] * T
    for n in range(T):
        row = [Fraction(v) for v in x[n]]
        mu = sum(row) / D
        var = sum((v - mu) ** 2 for v in row) / D
        r = 1.0 / math.sqrt(float(var + Fraction(eps)))
        m = seg_of[n]
        for d in range(D):
            xhat = float(row[d] - mu) * r
            y[n][d] = xhat * (1.0 + float(scale[m][d])) + float(shift[m][d])
        mean[n], rstd[n] = float(mu), r
    return y, mean, rstd


def _bf_backward(dy, x, scale, seg_of, nrows_mod, eps, per_token):
    T, D = len(x), len(x[0])
    dx = [[0.0] * D for _ in range(T)]
    dshift = [[0.0] * D for _ in range(nrows_mod)]
    dscale = [[0.0] * D for _ in range(nrows_mod)]
    for n in range(T):
        row = [Fraction(v) for v in x[n]]
        mu = sum(row) / D
        var = sum((v - mu) ** 2 for v in row) / D
        r = 1.0 / math.sqrt(float(var + Fraction(eps)))
        m = seg_of[n]
        xhat = [float(v - mu) * r for v in row]
        g = [float(dy[n][d]) * (1.0 + float(scale[m][d])) for d in range(D)]
        c1 = math.fsum(g) / D
        c2 = math.fsum(g[d] * xhat[d] for d in range(D)) / D
        for d in range(D):
            dx[n][d] = r * (g[d] - c1 - xhat[d] * c2)
            dshift[m][d] += float(dy[n][d])
            dscale[m][d] += float(dy[n][d]) * xhat[d]
    return dx, dshift, dscale


def _small_case(seed, lengths, D, per_token=False):
    rng = _rng(seed)
    T = int(sum(lengths))
    # dyadic values: exact in float32/float64 and as Fractions
    x = np.round(rng.normal(0.3, 1.5, (T, D)) * 64) / 64
    dy = np.round(rng.normal(0, 1, (T, D)) * 64) / 64
    rows = T if per_token else len(lengths)
    shift = np.round(rng.normal(0, 0.1, (rows, D)) * 256) / 256
    scale = np.round(rng.normal(0, 0.1, (rows, D)) * 256) / 256
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    if per_token:
        seg_of = list(range(T))
    else:
        seg_of = [m for m, L in enumerate(lengths) for _ in range(L)]
    return x, dy, shift, scale, cu, seg_of


@pin
def check_bruteforce(lib=None):
    for seed, lengths, D, per_token in [(1, (3,), 5, False), (2, (2, 0, 4), 8, False),
                                        (3, (1, 1), 2, False), (4, (4,), 7, True),
                                        (5, (2, 3), 3, True)]:
        x, dy, shift, scale, cu, seg_of = _small_case(seed, lengths, D, per_token)
        mod = oracle.PER_TOKEN if per_token else oracle.PER_SEGMENT
        eps = 1e-6
        for carrier in (np.float64, np.float32):
            xs, dys, shs, scs = (a.astype(carrier) for a in (x, dy, shift, scale))
            y, mean, rstd = oracle.forward(xs, shs, scs, eps, cu=cu, mod=mod, lib=lib)
            dx, dsh, dsc = oracle.backward(dys, xs, scs, eps, cu=cu, mod=mod, lib=lib)
            by, bmean, brstd = _bf_forward(x.tolist(), shift.tolist(), scale.tolist(), seg_of, eps)
            bdx, bdsh, bdsc = _bf_backward(dy.tolist(), x.tolist(), scale.tolist(), seg_of,
                                           shift.shape[0], eps, per_token)
            np.testing.assert_allclose(y, np.array(by), rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(mean, np.array(bmean), rtol=1e-13, atol=1e-15)
            np.testing.assert_allclose(rstd, np.array(brstd), rtol=1e-13)
            np.testing.assert_allclose(dx, np.array(bdx), rtol=1e-10, atol=1e-12)
            np.testing.assert_allclose(dsh, np.array(bdsh).reshape(dsh.shape), rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(dsc, np.array(bdsc).reshape(dsc.shape), rtol=1e-11, atol=1e-12)


def test_bruteforce():
    check_bruteforce()


# --------------------------------------------------------------------------------------------
# 2. closed form for D = 2 and the hand-derived golden case
# --------------------------------------------------------------------------------------------
@pin
def check_closed_form_d2(lib=None):
    # row (a, b), a != b: mu = (a+b)/2, var = ((a-b)/2)^2, xhat = +-1/sqrt(1 + eps/var)
    eps = 1e-6
    for a, b, sh, sc in [(1.0, 3.0, (0.25, -0.5), (0.5, -0.25)), (-7.5, 2.25, (0.0, 0.0), (0.0, 0.0)),
                         (1e3, 1e3 + 0.5, (1.0, 2.0), (-2.0, 3.0))]:
        x = np.array([[a, b]])
        y, mean, rstd = oracle.forward(x, np.array([sh]), np.array([sc]), eps, B=1, S=1, lib=lib)
        var = ((a - b) / 2) ** 2
        mag = 1.0 / math.sqrt(1.0 + eps / var)
        sgn = 1.0 if a > b else -1.0
        assert mean[0] == pytest.approx((a + b) / 2, rel=1e-15)
        assert rstd[0] == pytest.approx(1.0 / math.sqrt(var + eps), rel=1e-14)
        assert y[0, 0] == pytest.approx(sgn * mag * (1 + sc[0]) + sh[0], rel=1e-13)
        assert y[0, 1] == pytest.approx(-sgn * mag * (1 + sc[1]) + sh[1], rel=1e-13)


def test_closed_form_d2():
    check_closed_form_d2()


def _read_golden(name):
    path = os.path.join(os.path.dirname(__file__), "golden", name)
    rows = {}
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                key, *vals = line.split()
                rows[key] = [float(Fraction(v)) if "/" in v else float(v) for v in vals]
    return rows


def test_golden_hand_case():
    g = _read_golden("hand_case_d4.txt")
    x = np.array([g["x"]])
    y, mean, rstd = oracle.forward(x, np.array([g["shift"]]), np.array([g["scale"]]), g["eps"][0],
                                   B=1, S=1)
    assert mean[0] == pytest.approx(g["mean"][0], rel=1e-15)
    assert rstd[0] == pytest.approx(g["rstd"][0], rel=1e-14)
    np.testing.assert_allclose(y[0], g["y"], rtol=1e-13)
    dx, dsh, dsc = oracle.backward(np.array([g["dy"]]), x, np.array([g["scale"]]), g["eps"][0], B=1, S=1)
    np.testing.assert_allclose(dx[0], g["dx"], rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(dsh[0], g["dshift"], rtol=1e-15)
    np.testing.assert_allclose(dsc[0], g["dscale"], rtol=1e-13)


# --------------------------------------------------------------------------------------------
# 3. invariants
# --------------------------------------------------------------------------------------------
@pin
def check_unmodulated_rows_mean0_var(lib=None):
    # scale = shift = 0: every output row has mean 0 and variance var/(var+eps)
    rng = _rng(11)
    T, D, eps = 17, 96, 1e-6
    x = rng.normal(0.5, 2.0, (T, D)) * rng.uniform(1e-3, 1e2, (T, 1))
    z = np.zeros((1, D))
    y, mean, rstd = oracle.forward(x, z, z, eps, B=1, S=T, lib=lib)
    var = x.var(axis=1)                       # numpy's own biased variance
    np.testing.assert_allclose(y.mean(axis=1), 0.0, atol=1e-13)
    np.testing.assert_allclose(y.var(axis=1), var / (var + eps), rtol=1e-12)
    np.testing.assert_allclose(mean, x.mean(axis=1), rtol=1e-13)
    np.testing.assert_allclose(rstd, 1 / np.sqrt(var + eps), rtol=1e-12)
    # eps matters: with a larger eps the row variance drops accordingly
    y2, _, _ = oracle.forward(x, z, z, 0.5, B=1, S=T, lib=lib)
    np.testing.assert_allclose(y2.var(axis=1), var / (var + 0.5), rtol=1e-12)


def test_unmodulated_rows_mean0_var():
    check_unmodulated_rows_mean0_var()


@pin
def check_affine_covariance(lib=None):
    # LN(alpha*x + beta) with eps*alpha^2 equals sign(alpha) * LN(x) with eps
    rng = _rng(12)
    T, D, eps = 5, 40, 1e-3
    x = rng.normal(0, 1, (T, D))
    z = np.zeros((1, D))
    y0, _, r0 = oracle.forward(x, z, z, eps, B=1, S=T, lib=lib)
    for alpha, beta in [(3.0, -7.0), (-0.25, 100.0)]:
        y1, m1, r1 = oracle.forward(alpha * x + beta, z, z, eps * alpha * alpha, B=1, S=T, lib=lib)
        np.testing.assert_allclose(y1, math.copysign(1, alpha) * y0, rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(r1, r0 / abs(alpha), rtol=1e-11)


def test_affine_covariance():
    check_affine_covariance()


@pin
def check_shift_scale_linearity(lib=None):
    rng = _rng(13)
    B, S, D, eps = 3, 4, 24, 1e-6
    x = rng.normal(0, 1, (B * S, D))
    sh1, sh2 = rng.normal(0, 0.1, (B, D)), rng.normal(0, 0.3, (B, D))
    sc1, sc2 = rng.normal(0, 0.1, (B, D)), rng.normal(0, 0.3, (B, D))
    z = np.zeros((B, D))
    y11, _, _ = oracle.forward(x, sh1, sc1, eps, B=B, S=S, lib=lib)
    y21, _, _ = oracle.forward(x, sh1 + sh2, sc1, eps, B=B, S=S, lib=lib)
    y12, _, _ = oracle.forward(x, sh1, sc1 + sc2, eps, B=B, S=S, lib=lib)
    xhat, _, _ = oracle.forward(x, z, z, eps, B=B, S=S, lib=lib)
    # adding shift2 adds exactly shift2 of the token's own sample
    np.testing.assert_allclose(y21 - y11, np.repeat(sh2, S, axis=0), atol=1e-13)
    # dy/dscale = xhat, per sample
    np.testing.assert_allclose(y12 - y11, xhat * np.repeat(sc2, S, axis=0), atol=1e-13)
    # scale = -1 kills the normalised part entirely
    ym, _, _ = oracle.forward(x, sh1, -np.ones((B, D)), eps, B=B, S=S, lib=lib)
    np.testing.assert_allclose(ym, np.repeat(sh1, S, axis=0), atol=1e-15)


def test_shift_scale_linearity():
    check_shift_scale_linearity()


@pin
def check_dshift_is_token_sum_of_dy(lib=None):
    rng = _rng(14)
    lengths = (5, 0, 9, 1)
    D = 33
    T = sum(lengths)
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    x = rng.normal(0, 1, (T, D))
    dy = rng.normal(0, 1, (T, D))
    scale = rng.normal(0, 0.1, (len(lengths), D))
    _, dsh, dsc = oracle.backward(dy, x, scale, cu=cu, lib=lib)
    z = np.zeros((len(lengths), D))
    xhat, _, _ = oracle.forward(x, z, z, cu=cu, lib=lib)
    for m in range(len(lengths)):
        sl = slice(cu[m], cu[m + 1])
        np.testing.assert_allclose(dsh[m], dy[sl].sum(axis=0), rtol=1e-13, atol=1e-14)
        np.testing.assert_allclose(dsc[m], (dy[sl] * xhat[sl]).sum(axis=0), rtol=1e-12, atol=1e-13)
    assert np.all(dsh[1] == 0) and np.all(dsc[1] == 0)          # empty segment
    # dshift does not depend on x or scale
    _, dsh2, _ = oracle.backward(dy, rng.normal(3, 5, (T, D)), 5 * scale, cu=cu, lib=lib)
    np.testing.assert_allclose(dsh2, dsh, rtol=1e-15)


def test_dshift_is_token_sum_of_dy():
    check_dshift_is_token_sum_of_dy()


@pin
def check_dx_invariants(lib=None):
    # sum_d dx = 0 and sum_d dx*xhat = r*D*c2*eps/(var+eps) (which is ~0)
    rng = _rng(15)
    T, D, eps = 9, 64, 1e-2          # big eps so the second identity is not trivially 0
    x = rng.normal(0.5, 2, (T, D))
    dy = rng.normal(0, 1, (T, D))
    scale = rng.normal(0, 0.1, (1, D))
    dx, _, _ = oracle.backward(dy, x, scale, eps, B=1, S=T, lib=lib)
    z = np.zeros((1, D))
    xhat, _, rstd = oracle.forward(x, z, z, eps, B=1, S=T, lib=lib)
    g = dy * (1 + scale)
    c2 = (g * xhat).mean(axis=1)
    var = x.var(axis=1)
    np.testing.assert_allclose(dx.sum(axis=1), 0, atol=1e-12)
    np.testing.assert_allclose((dx * xhat).sum(axis=1), rstd * D * c2 * eps / (var + eps), rtol=1e-9, atol=1e-13)


def test_dx_invariants():
    check_dx_invariants()


# --------------------------------------------------------------------------------------------
# 4. library routine: torch layer_norm + autograd in float64
# --------------------------------------------------------------------------------------------
@pin
def check_against_torch_layer_norm_autograd(lib=None):
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    rng = _rng(16)
    for B, S, D, per_token in [(2, 7, 48, False), (1, 5, 130, True), (3, 1, 16, False)]:
        T = B * S
        eps = 1e-6
        x = rng.normal(0.5, 2, (T, D))
        dy = rng.normal(0, 1, (T, D))
        rows = T if per_token else B
        shift = rng.normal(0, 0.1, (rows, D))
        scale = rng.normal(0, 0.1, (rows, D))
        mod = oracle.PER_TOKEN if per_token else oracle.PER_SEGMENT
        y, mean, rstd = oracle.forward(x, shift, scale, eps, B=B, S=S, mod=mod, lib=lib)
        dx, dsh, dsc = oracle.backward(dy, x, scale, eps, B=B, S=S, mod=mod, lib=lib)

        tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
        tsh = torch.tensor(shift, dtype=torch.float64, requires_grad=True)
        tsc = torch.tensor(scale, dtype=torch.float64, requires_grad=True)
        ln = F.layer_norm(tx, (D,), eps=eps)
        if per_token:
            ty = ln * (1 + tsc) + tsh
        else:
            ty = (ln.view(B, S, D) * (1 + tsc[:, None, :]) + tsh[:, None, :]).view(T, D)
        ty.backward(torch.tensor(dy, dtype=torch.float64))
        np.testing.assert_allclose(y, ty.detach().numpy(), rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-8, atol=1e-11)
        np.testing.assert_allclose(dsh, tsh.grad.numpy(), rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(dsc, tsc.grad.numpy(), rtol=1e-9, atol=1e-11)
        # scale = shift = 0 reduces to the library routine itself
        z = np.zeros_like(shift)
        y0, _, _ = oracle.forward(x, z, z, eps, B=B, S=S, mod=mod, lib=lib)
        np.testing.assert_allclose(y0, ln.detach().numpy(), rtol=1e-10, atol=1e-12)


def test_against_torch_layer_norm_autograd():
    check_against_torch_layer_norm_autograd()


# --------------------------------------------------------------------------------------------
# 5. finite differences of L = sum(dy * y)
# --------------------------------------------------------------------------------------------
@pin
def check_finite_differences(lib=None):
    rng = _rng(17)
    B, S, D, eps = 2, 3, 12, 1e-6
    T = B * S
    x = rng.normal(0.5, 2, (T, D))
    dy = rng.normal(0, 1, (T, D))
    shift = rng.normal(0, 0.1, (B, D))
    scale = rng.normal(0, 0.1, (B, D))

    def loss(x_, sh_, sc_):
        y, _, _ = oracle.forward(x_, sh_, sc_, eps, B=B, S=S, lib=lib)
        return float((dy * y).sum())

    dx, dsh, dsc = oracle.backward(dy, x, scale, eps, B=B, S=S, lib=lib)
    h = 1e-5
    for arr, grad, which in [(x, dx, 0), (shift, dsh, 1), (scale, dsc, 2)]:
        num = np.zeros_like(arr)
        for idx in np.ndindex(arr.shape):
            args = [x, shift, scale]
            p, m = arr.copy(), arr.copy()
            p[idx] += h
            m[idx] -= h
            args[which] = p
            lp = loss(*args)
            args[which] = m
            lm = loss(*args)
            num[idx] = (lp - lm) / (2 * h)
        np.testing.assert_allclose(grad, num, rtol=2e-6, atol=2e-8)


def test_finite_differences():
    check_finite_differences()


def test_finite_differences_config0_row():
    # one row of the tiny-fp32 workload's width (D=1536), sampled coordinates
    rng = _rng(18)
    D, eps = 1536, 1e-6
    x = rng.normal(0, 1, (1, D))
    dy = rng.normal(0, 1, (1, D))
    shift = rng.normal(0, 0.1, (1, D))
    scale = rng.normal(0, 0.1, (1, D))
    dx, _, dsc = oracle.backward(dy, x, scale, eps, B=1, S=1)
    h = 1e-5
    for d in rng.choice(D, 12, replace=False):
        p, m = x.copy(), x.copy()
        p[0, d] += h
        m[0, d] -= h
        lp = (dy * oracle.forward(p, shift, scale, eps, B=1, S=1)[0]).sum()
        lm = (dy * oracle.forward(m, shift, scale, eps, B=1, S=1)[0]).sum()
        assert dx[0, d] == pytest.approx((lp - lm) / (2 * h), rel=1e-5, abs=1e-8)


# --------------------------------------------------------------------------------------------
# 6. structure: varlen == per-segment calls, per-token == broadcast, degenerate rows
# --------------------------------------------------------------------------------------------
@pin
def check_varlen_equals_per_segment_calls(lib=None):
    rng = _rng(19)
    lengths = (4, 0, 7, 1, 3)
    D = 20
    T = sum(lengths)
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    x = rng.normal(0, 1, (T, D))
    dy = rng.normal(0, 1, (T, D))
    shift = rng.normal(0, 0.1, (len(lengths), D))
    scale = rng.normal(0, 0.1, (len(lengths), D))
    y, mean, rstd = oracle.forward(x, shift, scale, cu=cu, lib=lib)
    dx, dsh, dsc = oracle.backward(dy, x, scale, cu=cu, lib=lib)
    for m, L in enumerate(lengths):
        sl = slice(cu[m], cu[m + 1])
        if L == 0:
            assert np.all(dsh[m] == 0) and np.all(dsc[m] == 0)
            continue
        ym, mm, rm = oracle.forward(x[sl], shift[m:m + 1], scale[m:m + 1], B=1, S=L, lib=lib)
        dxm, dshm, dscm = oracle.backward(dy[sl], x[sl], scale[m:m + 1], B=1, S=L, lib=lib)
        assert np.array_equal(y[sl], ym) and np.array_equal(mean[sl], mm) and np.array_equal(rstd[sl], rm)
        assert np.array_equal(dx[sl], dxm)
        assert np.array_equal(dsh[m], dshm[0]) and np.array_equal(dsc[m], dscm[0])
    # a fixed-length batch is the varlen call with uniform offsets
    B, S = 3, 5
    x = rng.normal(0, 1, (B * S, D))
    sh, sc = rng.normal(0, 0.1, (B, D)), rng.normal(0, 0.1, (B, D))
    ya, _, _ = oracle.forward(x, sh, sc, B=B, S=S, lib=lib)
    for b in range(B):
        yb, _, _ = oracle.forward(x[b * S:(b + 1) * S], sh[b:b + 1], sc[b:b + 1], B=1, S=S, lib=lib)
        assert np.array_equal(ya[b * S:(b + 1) * S], yb)


def test_varlen_equals_per_segment_calls():
    check_varlen_equals_per_segment_calls()


@pin
def check_per_token_equals_broadcast(lib=None):
    rng = _rng(20)
    B, S, D = 2, 6, 28
    T = B * S
    x = rng.normal(0, 1, (T, D))
    dy = rng.normal(0, 1, (T, D))
    shift = rng.normal(0, 0.1, (B, D))
    scale = rng.normal(0, 0.1, (B, D))
    y, mean, rstd = oracle.forward(x, shift, scale, B=B, S=S, lib=lib)
    dx, dsh, dsc = oracle.backward(dy, x, scale, B=B, S=S, lib=lib)
    sh_t, sc_t = np.repeat(shift, S, axis=0), np.repeat(scale, S, axis=0)
    yt, mt, rt = oracle.forward(x, sh_t, sc_t, B=B, S=S, mod=oracle.PER_TOKEN, lib=lib)
    dxt, dsht, dsct = oracle.backward(dy, x, sc_t, B=B, S=S, mod=oracle.PER_TOKEN, lib=lib)
    assert np.array_equal(y, yt) and np.array_equal(mean, mt) and np.array_equal(rstd, rt)
    assert np.array_equal(dx, dxt)
    assert np.array_equal(dsht, dy)
    np.testing.assert_allclose(dsht.reshape(B, S, D).sum(axis=1), dsh, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(dsct.reshape(B, S, D).sum(axis=1), dsc, rtol=1e-12, atol=1e-13)


def test_per_token_equals_broadcast():
    check_per_token_equals_broadcast()


@pin
def check_degenerate_rows(lib=None):
    # constant row: var = 0, r = 1/sqrt(eps) = 1000, xhat = 0, y = shift; no NaN.  dx is NOT 0:
    # with xhat = 0 the Jacobian is r*(I - 1/D), so dx = 1000*(g - mean(g))
    D, eps = 16, 1e-6
    x = np.full((2, D), 3.25)
    x[1] = np.arange(D)
    shift = np.linspace(-1, 1, D)[None]
    scale = np.linspace(0.5, -0.5, D)[None]
    dy = np.ones((2, D)) * np.arange(1, D + 1)
    y, mean, rstd = oracle.forward(x, shift, scale, eps, B=1, S=2, lib=lib)
    dx, dsh, dsc = oracle.backward(dy, x, scale, eps, B=1, S=2, lib=lib)
    assert rstd[0] == pytest.approx(1000.0, rel=1e-14) and mean[0] == 3.25
    assert np.array_equal(y[0], shift[0])
    g0 = dy[0] * (1 + scale[0])
    np.testing.assert_allclose(dx[0], 1000.0 * (g0 - g0.mean()), rtol=1e-12, atol=1e-9)
    assert np.array_equal(dsh[0], dy.sum(axis=0))
    assert np.all(np.isfinite(y)) and np.all(np.isfinite(dx))
    # non-finite input propagates to its own row only
    x[0, 3] = np.inf
    y, _, _ = oracle.forward(x, shift, scale, eps, B=1, S=2, lib=lib)
    assert not np.all(np.isfinite(y[0])) and np.all(np.isfinite(y[1]))


def test_degenerate_rows():
    check_degenerate_rows()


def test_bad_arguments():
    x = np.zeros((4, 8))
    z = np.zeros((1, 8))
    with pytest.raises(ValueError):
        oracle.forward(x, z, z, cu=np.array([0, 3]))            # offsets do not end at T
    with pytest.raises(RuntimeError):
        oracle.forward(x, np.zeros((2, 8)), np.zeros((2, 8)), cu=np.array([0, 5, 4]))   # decreasing
    with pytest.raises(RuntimeError):
        oracle.forward(x, z, z, B=1, S=4, mod=7)


def test_variance_is_two_pass_stable():
    # huge common offset: E[x^2]-mu^2 would lose everything, the two-pass form does not
    rng = _rng(21)
    D = 512
    base = rng.normal(0, 1, (1, D))
    x = base + 1e8
    z = np.zeros((1, D))
    _, _, r = oracle.forward(x, z, z, 1e-6, B=1, S=1)
    var = np.var(x.astype(np.longdouble))                        # x itself is rounded at 1e8
    assert r[0] == pytest.approx(float(1 / np.sqrt(var + 1e-6)), rel=1e-9)


def test_threads_do_not_change_results():
    rng = _rng(22)
    B, S, D = 2, 37, 200
    x = rng.normal(0, 1, (B * S, D)).astype(np.float32)
    dy = rng.normal(0, 1, (B * S, D)).astype(np.float32)
    sh = rng.normal(0, 0.1, (B, D)).astype(np.float32)
    sc = rng.normal(0, 0.1, (B, D)).astype(np.float32)
    n0 = oracle.num_threads()
    try:
        oracle.set_num_threads(1)
        a = oracle.forward(x, sh, sc, B=B, S=S) + oracle.backward(dy, x, sc, B=B, S=S)
        oracle.set_num_threads(max(2, n0))
        b = oracle.forward(x, sh, sc, B=B, S=S) + oracle.backward(dy, x, sc, B=B, S=S)
    finally:
        oracle.set_num_threads(n0)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)
