"""Pins for the float64 oracle of the gated-residual + LayerNorm-Modulate operator
(oracle/gated_oracle.c): everything here checks it against something that is not itself --
literal loops with exact rationals, the composition of a plain numpy residual step with the
separately pinned LayerNorm-Modulate oracle, torch's float64 layer_norm + autograd (a library
routine), finite differences, and the storage rounding against numpy's / torch's own casts.
The last test plants mistakes in a copy of the C source and requires a pin to notice each.

The paper only names this fusion ("Gate + Norm", Sec. 4.4); the definition is the DiT block's:
h = x + gate*u stored in the I/O type, then y = LN(h)*(1+scale)+shift (Sec. 3.3 for that part).
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from oracle import gated_oracle as go

PIN_FUNCS = []


def pin(f):
    PIN_FUNCS.append(f)
    return f


def _rng(seed):
    return np.random.default_rng(seed)


def _case(seed, lengths, D, dtype=np.float64):
    rng = _rng(seed)
    T, nseg = int(sum(lengths)), len(lengths)
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    c = dict(
        x=rng.normal(0.3, 1.5, (T, D)), u=rng.normal(0, 1, (T, D)),
        gate=rng.normal(0, 0.5, (nseg, D)), shift=rng.normal(0, 0.3, (nseg, D)),
        scale=rng.normal(0, 0.3, (nseg, D)), dy=rng.normal(0, 1, (T, D)), dh=rng.normal(0, 1, (T, D)))
    c = {k: v.astype(dtype) for k, v in c.items()}
    c.update(cu=cu, T=T, D=D, nseg=nseg, seg_of=np.repeat(np.arange(nseg), lengths))
    return c


# --------------------------------------------------------------------------------------------
# 1. literal loops with exact rationals on a tiny case (forward and backward)
# --------------------------------------------------------------------------------------------
@pin
def test_bruteforce_tiny(lib=None):
    c = _case(1, [2, 0, 3], 5)
    eps = 1e-3
    h, y, mean, rstd = go.forward(c["x"], c["u"], c["gate"], c["shift"], c["scale"], eps, cu=c["cu"], lib=lib)
    dx, du, dgate, dshift, dscale = go.backward(c["dy"], c["dh"], h, c["u"], c["gate"], c["scale"], eps,
                                                cu=c["cu"], lib=lib)
    T, D, nseg = c["T"], c["D"], c["nseg"]
    F = Fraction
    eg = [[F(0)] * D for _ in range(nseg)]
    es = [[F(0)] * D for _ in range(nseg)]
    ec = [[0.0] * D for _ in range(nseg)]
    for n in range(T):
        m = int(c["seg_of"][n])
        hr = [F(float(c["x"][n, d])) + F(float(c["gate"][m, d])) * F(float(c["u"][n, d])) for d in range(D)]
        mu = sum(hr) / D
        var = sum((v - mu) ** 2 for v in hr) / D
        r = 1.0 / math.sqrt(float(var + F(eps)))
        assert mean[n] == pytest.approx(float(mu), rel=1e-13, abs=1e-15)
        assert rstd[n] == pytest.approx(r, rel=1e-13)
        hhat = [float(v - mu) * r for v in hr]
        g = [float(c["dy"][n, d]) * (1.0 + float(c["scale"][m, d])) for d in range(D)]
        c1 = sum(g) / D
        c2 = sum(g[d] * hhat[d] for d in range(D)) / D
        for d in range(D):
            assert h[n, d] == pytest.approx(float(hr[d]), rel=1e-14, abs=1e-300)
            assert y[n, d] == pytest.approx(hhat[d] * (1.0 + c["scale"][m, d]) + c["shift"][m, d], rel=1e-11, abs=1e-12)
            e_dx = float(c["dh"][n, d]) + r * (g[d] - c1 - hhat[d] * c2)
            assert dx[n, d] == pytest.approx(e_dx, rel=1e-10, abs=1e-11)
            assert du[n, d] == pytest.approx(float(c["gate"][m, d]) * e_dx, rel=1e-10, abs=1e-11)
            eg[m][d] += F(float(c["u"][n, d])) * F(e_dx)
            es[m][d] += F(float(c["dy"][n, d]))
            ec[m][d] += float(c["dy"][n, d]) * hhat[d]
    for m in range(nseg):
        for d in range(D):
            assert dgate[m, d] == pytest.approx(float(eg[m][d]), rel=1e-9, abs=1e-10)
            assert dshift[m, d] == pytest.approx(float(es[m][d]), rel=1e-12, abs=1e-13)
            assert dscale[m, d] == pytest.approx(ec[m][d], rel=1e-9, abs=1e-10)
    assert np.all(dgate[1] == 0) and np.all(dshift[1] == 0) and np.all(dscale[1] == 0)   # empty segment


# --------------------------------------------------------------------------------------------
# 2. composition with the separately pinned LayerNorm-Modulate oracle
# --------------------------------------------------------------------------------------------
@pin
def test_is_residual_then_lnmod(lib=None):
    c = _case(2, [7, 1, 12], 48)
    h, y, mean, rstd = go.forward(c["x"], c["u"], c["gate"], c["shift"], c["scale"], cu=c["cu"], lib=lib)
    h_np = c["x"] + c["gate"][c["seg_of"]] * c["u"]
    assert np.allclose(h, h_np, rtol=1e-15, atol=0)
    y2, m2, r2 = oracle.forward(h_np, c["shift"], c["scale"], cu=c["cu"])
    assert np.allclose(y, y2, rtol=1e-12, atol=1e-13)
    assert np.allclose(mean, m2, rtol=1e-13, atol=1e-15) and np.allclose(rstd, r2, rtol=1e-13)
    dx, du, dgate, dshift, dscale = go.backward(c["dy"], c["dh"], h, c["u"], c["gate"], c["scale"], cu=c["cu"], lib=lib)
    dln, dsh2, dsc2 = oracle.backward(c["dy"], h_np, c["scale"], cu=c["cu"])
    assert np.allclose(dx, c["dh"] + dln, rtol=1e-11, atol=1e-12)
    assert np.allclose(du, c["gate"][c["seg_of"]] * (c["dh"] + dln), rtol=1e-11, atol=1e-12)
    assert np.allclose(dshift, dsh2, rtol=1e-12, atol=1e-12) and np.allclose(dscale, dsc2, rtol=1e-11, atol=1e-11)
    eg = np.zeros_like(dgate)
    np.add.at(eg, c["seg_of"], c["u"] * (c["dh"] + dln))
    assert np.allclose(dgate, eg, rtol=1e-10, atol=1e-11)


@pin
def test_zero_gate_is_plain_lnmod(lib=None):
    c = _case(3, [9, 4], 32)
    z = np.zeros_like(c["gate"])
    h, y, mean, rstd = go.forward(c["x"], c["u"], z, c["shift"], c["scale"], cu=c["cu"], lib=lib)
    assert np.array_equal(h, c["x"])
    y2, _, _ = oracle.forward(c["x"], c["shift"], c["scale"], cu=c["cu"])
    assert np.allclose(y, y2, rtol=1e-12, atol=1e-13)
    dx, du, dgate, _, _ = go.backward(c["dy"], c["dh"], h, c["u"], z, c["scale"], cu=c["cu"], lib=lib)
    assert np.all(du == 0)
    assert np.abs(dgate).max() > 0.1            # the gate still receives a gradient


# --------------------------------------------------------------------------------------------
# 3. library routine: torch float64 layer_norm + autograd
# --------------------------------------------------------------------------------------------
@pin
def test_against_torch_autograd(lib=None):
    c = _case(4, [6, 10, 3], 40)
    eps = 1e-5
    seg = torch.from_numpy(c["seg_of"])
    t = {k: torch.tensor(c[k], dtype=torch.float64, requires_grad=k in ("x", "u", "gate", "shift", "scale"))
         for k in ("x", "u", "gate", "shift", "scale", "dy", "dh")}
    h_t = t["x"] + t["gate"][seg] * t["u"]
    y_t = torch.nn.functional.layer_norm(h_t, (c["D"],), eps=eps) * (1 + t["scale"][seg]) + t["shift"][seg]
    ((t["dy"] * y_t).sum() + (t["dh"] * h_t).sum()).backward()
    h, y, _, _ = go.forward(c["x"], c["u"], c["gate"], c["shift"], c["scale"], eps, cu=c["cu"], lib=lib)
    dx, du, dgate, dshift, dscale = go.backward(c["dy"], c["dh"], h, c["u"], c["gate"], c["scale"], eps,
                                                cu=c["cu"], lib=lib)
    assert np.allclose(h, h_t.detach().numpy(), rtol=1e-14, atol=0)
    assert np.allclose(y, y_t.detach().numpy(), rtol=1e-10, atol=1e-11)
    for got, name in ((dx, "x"), (du, "u"), (dgate, "gate"), (dshift, "shift"), (dscale, "scale")):
        assert np.allclose(got, t[name].grad.numpy(), rtol=1e-9, atol=1e-10), name


# --------------------------------------------------------------------------------------------
# 4. finite differences of L = sum(dy*y) + sum(dh*h) through the oracle's own forward
# --------------------------------------------------------------------------------------------
@pin
def test_finite_differences(lib=None):
    c = _case(5, [3, 4], 12)
    eps = 1e-4

    def loss(x, u, gate):
        h, y, _, _ = go.forward(x, u, gate, c["shift"], c["scale"], eps, cu=c["cu"], lib=lib)
        return float((c["dy"] * y).sum() + (c["dh"] * h).sum())

    h, _, _, _ = go.forward(c["x"], c["u"], c["gate"], c["shift"], c["scale"], eps, cu=c["cu"], lib=lib)
    dx, du, dgate, _, _ = go.backward(c["dy"], c["dh"], h, c["u"], c["gate"], c["scale"], eps, cu=c["cu"], lib=lib)
    rng = _rng(50)
    step = 1e-6
    for name, grad in (("x", dx), ("u", du), ("gate", dgate)):
        base = c[name]
        for _ in range(12):
            idx = tuple(int(rng.integers(0, s)) for s in base.shape)
            args = {k: c[k].copy() for k in ("x", "u", "gate")}
            args[name][idx] = base[idx] + step
            up = loss(**args)
            args[name][idx] = base[idx] - step
            dn = loss(**args)
            assert (up - dn) / (2 * step) == pytest.approx(grad[idx], rel=2e-6, abs=2e-7), (name, idx)


# --------------------------------------------------------------------------------------------
# 5. the storage rounding of h
# --------------------------------------------------------------------------------------------
@pin
def test_storage_rounding(lib=None):
    c = _case(6, [5, 6], 64, dtype=np.float32)
    exact = c["x"].astype(np.float64) + c["gate"].astype(np.float64)[c["seg_of"]] * c["u"].astype(np.float64)
    h0, _, _, _ = go.forward(c["x"], c["u"], c["gate"], c["shift"], c["scale"], cu=c["cu"], lib=lib)
    assert np.array_equal(h0, exact)                             # no rounding: float64 holds it exactly
    h1, y1, m1, r1 = go.forward(c["x"], c["u"], c["gate"], c["shift"], c["scale"], cu=c["cu"],
                                quant=go.QUANT_F32, lib=lib)
    f32 = exact.astype(np.float32)                                # numpy casts to nearest even
    assert np.array_equal(h1, f32.astype(np.float64))
    h2, y2, m2, r2 = go.forward(c["x"], c["u"], c["gate"], c["shift"], c["scale"], cu=c["cu"],
                                quant=go.QUANT_BF16, lib=lib)
    bf = torch.from_numpy(f32).to(torch.bfloat16).to(torch.float64).numpy()    # torch rounds to nearest even
    assert np.array_equal(h2, bf)
    assert not np.array_equal(h2, h1)
    # the LayerNorm sees the stored values
    ye, me, re = oracle.forward(bf, c["shift"], c["scale"], cu=c["cu"])
    assert np.allclose(y2, ye, rtol=1e-12, atol=1e-13) and np.allclose(m2, me, rtol=1e-13, atol=1e-15)
    # ties go to even, and a float32 tie is decided before the bf16 one
    x = np.array([[1.0, 1.0, 1.0, 1.0]], dtype=np.float32)
    u = np.array([[2.0 ** -8, 3 * 2.0 ** -8, 2.0 ** -8 + 2.0 ** -30, 2.0 ** -9]], dtype=np.float32)
    one = np.ones((1, 4), dtype=np.float32)
    zero = np.zeros((1, 4), dtype=np.float32)
    hq, _, _, _ = go.forward(x, u, one, zero, zero, B=1, S=1, quant=go.QUANT_BF16, lib=lib)
    assert hq[0].tolist() == [1.0, 1.0 + 2.0 ** -6, 1.0, 1.0]


@pin
def test_bad_arguments(lib=None):
    x = np.zeros((4, 8))
    z = np.zeros((2, 8))
    with pytest.raises(ValueError):
        go.forward(x, x, z, z, z, cu=np.array([0, 3, 5]), lib=lib)
    with pytest.raises(RuntimeError):
        go.forward(x, x, np.zeros((3, 8)), np.zeros((3, 8)), np.zeros((3, 8)), cu=np.array([0, 5, 2, 4]), lib=lib)
    with pytest.raises(RuntimeError):
        go.forward(x, x, z, z, z, B=2, S=2, quant=3, lib=lib)


# --------------------------------------------------------------------------------------------
# 6. planted mistakes: (label, text to find, replacement, occurrence)
# --------------------------------------------------------------------------------------------
MUTANTS = [
    ("gate term subtracted", "const double t = ld(x, in_f32, n * D + d)\n                                 + ld(gate",
     "const double t = ld(x, in_f32, n * D + d)\n                                 - ld(gate", 0),
    ("gate row of the wrong segment", "ld(gate, in_f32, m * D + d) * ld(u, in_f32, n * D + d);",
     "ld(gate, in_f32, 0 * D + d) * ld(u, in_f32, n * D + d);", 0),
    ("statistics of x instead of h", "row_stats(h + n * D, D, eps, &mu, &r);",
     "{ double tmp[4096]; for (int64_t d = 0; d < D; ++d) tmp[d] = ld(x, in_f32, n * D + d); row_stats(tmp, D, eps, &mu, &r); }", 0),
    ("unbiased variance", "*r_out = 1.0 / sqrt(q / (double)D + eps);", "*r_out = 1.0 / sqrt(q / (double)(D - 1) + eps);", 0),
    ("eps outside the sqrt (backward)", "r[n] = 1.0 / sqrt(q / (double)D + eps);", "r[n] = 1.0 / (sqrt(q / (double)D) + eps);", 0),
    ("h not rounded to bf16", "if (quant == 2) f = to_bf16(f);", "if (quant == 3) f = to_bf16(f);", 0),
    ("bf16 by truncation", "u += 0x7fffu + ((u >> 16) & 1u);", "u += 0u;", 0),
    ("bf16 ties away from zero", "u += 0x7fffu + ((u >> 16) & 1u);", "u += 0x8000u;", 0),
    ("dx forgets the residual gradient", "dx[n * D + d] = ld(dh, in_f32, n * D + d) + dln;", "dx[n * D + d] = dln;", 0),
    ("du from the LayerNorm part only", "du[n * D + d] = ld(gate, in_f32, m * D + d) * dx[n * D + d];",
     "du[n * D + d] = ld(gate, in_f32, m * D + d) * dln;", 0),
    ("du without the gate", "du[n * D + d] = ld(gate, in_f32, m * D + d) * dx[n * D + d];", "du[n * D + d] = dx[n * D + d];", 0),
    ("dgate sums dx only", "dgate[m * D + d] += ld(u, in_f32, n * D + d) * dx[n * D + d];", "dgate[m * D + d] += dx[n * D + d];", 0),
    ("dgate uses du", "dgate[m * D + d] += ld(u, in_f32, n * D + d) * dx[n * D + d];",
     "dgate[m * D + d] += ld(u, in_f32, n * D + d) * du[n * D + d];", 0),
    ("c2 term dropped", "const double dln = r[n] * (g - c1 - hhat * c2);", "const double dln = r[n] * (g - c1);", 0),
    ("c1 term sign", "const double dln = r[n] * (g - c1 - hhat * c2);", "const double dln = r[n] * (g + c1 - hhat * c2);", 0),
    ("g without 1+scale", "const double g = ld(dy, in_f32, n * D + d) * (1.0 + ld(scale, in_f32, m * D + d));",
     "const double g = ld(dy, in_f32, n * D + d);", 1),
    ("dscale sums dy only", "dscale[m * D + d] += t * hhat;", "dscale[m * D + d] += t;", 0),
    ("token sums skip the last token", "for (int64_t n = n0; n < n1; ++n) {\n                for (int64_t d = d0; d < d1; ++d) {\n                    const double t",
     "for (int64_t n = n0; n < n1 - 1; ++n) {\n                for (int64_t d = d0; d < d1; ++d) {\n                    const double t", 0),
    ("forward: scale instead of 1+scale", "y[n * D + d] = hhat * (1.0 + ld(scale", "y[n * D + d] = hhat * (ld(scale", 0),
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
    with open(go.SOURCE) as f:
        src = f.read()
    mutated = _replace_nth(src, old, new, nth)
    assert mutated != src
    c_path = os.path.join(tmp_path, "mutant.c")
    with open(c_path, "w") as f:
        f.write(mutated)
    lib = go.load(go.build(force=True, source=c_path, output=os.path.join(tmp_path, "libmutant.so")))
    caught = []
    for check in PIN_FUNCS:
        try:
            check(lib)
        except AssertionError:
            caught.append(check.__name__)
    assert caught, "no pin notices the planted mistake: " + label


def test_unmutated_source_passes_every_pin(tmp_path):
    lib = go.load(go.build(force=True, source=go.SOURCE, output=os.path.join(tmp_path, "libclean.so")))
    for check in PIN_FUNCS:
        check(lib)
