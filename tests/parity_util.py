"""Comparison helpers for the GPU-vs-oracle parity tests.

Tolerances (stated by the workload definition: bf16 I/O max abs 2e-2 and relative L2 4e-3;
fp32 I/O 1e-5 relative; mean/rstd 1e-5 relative), read as follows:

  bf16 tensors   rel-L2 <= 4e-3 and, element by element, |err| <= 2e-2 + 2^-8 |ref|: the plain
                 2e-2 bound cannot hold where |ref| >= 8, because rounding the exact result to
                 bf16 already moves it by up to 2^-9 |ref| there.  In addition every GPU value
                 must lie within one bf16 ulp of the correctly rounded reference, plus the
                 fp32-level absolute slack 1e-5 max|ref| (a value that cancellation made tiny,
                 such as a dx entry near zero, carries the absolute fp32 error of its operands,
                 which can exceed the ulp of the tiny result).
  fp32 tensors   rel-L2 <= 1e-5 and max|err| <= 1e-5 max|ref| (also used for the float32
                 dshift/dscale sums of the bf16 workloads).
  rstd           element-wise relative error <= 1e-5.
  mean           |err| <= 1e-5 max(|mean_ref|, std_ref): a pure relative bound is ill-posed for
                 rows whose mean happens to be near zero.
"""
import numpy as np
import torch


def to_device(a, dtype, device="cuda"):
    """float32 host array (already exact in `dtype`) -> device tensor of that dtype."""
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype == "bf16":
        return t.to(torch.bfloat16).to(device)
    return t.to(device)


def to_host64(t):
    return t.detach().to("cpu").to(torch.float64).numpy()


def rel_l2(got, ref):
    den = float(np.linalg.norm(ref.ravel()))
    num = float(np.linalg.norm((got - ref).ravel()))
    return num / den if den > 0 else num


def bf16_round(a64):
    """Correctly rounded (nearest even) bf16 value of float64 data, as float64.  Rounds from
    float64 in one step (via the float32 value and a sticky correction is not needed: torch
    rounds double -> bfloat16 directly)."""
    return torch.from_numpy(np.ascontiguousarray(a64)).to(torch.bfloat16).to(torch.float64).numpy()


def bf16_ulp(a64):
    a = np.abs(a64)
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -126)))
    return 2.0 ** (e - 7)


def check_io_tensor(name, got_t, ref64, dtype):
    got = to_host64(got_t).reshape(ref64.shape)
    assert np.all(np.isfinite(got)), name + ": non-finite values"
    err = np.abs(got - ref64)
    if dtype == "bf16":
        r = rel_l2(got, ref64)
        assert r <= 4e-3, "%s: rel-L2 %.3e > 4e-3" % (name, r)
        bound = 2e-2 + 2.0 ** -8 * np.abs(ref64)
        bad = err > bound
        assert not bad.any(), "%s: %d elements beyond 2e-2 + 2^-8|ref| (worst %.3e at |ref| %.3e)" % (
            name, int(bad.sum()), float(err.max()), float(np.abs(ref64).ravel()[err.argmax()]))
        rounded = bf16_round(ref64)
        ulp = bf16_ulp(rounded)
        off = np.abs(got - rounded) > ulp * 1.0001 + 1e-5 * float(np.abs(ref64).max())
        assert not off.any(), "%s: %d elements more than one bf16 ulp from the rounded reference" % (
            name, int(off.sum()))
    else:
        check_f32_tensor(name, got, ref64)
    return float(err.max())


def check_f32_tensor(name, got, ref64, rel=1e-5):
    if isinstance(got, torch.Tensor):
        got = to_host64(got)
    got = got.reshape(ref64.shape)
    assert np.all(np.isfinite(got)), name + ": non-finite values"
    r = rel_l2(got, ref64)
    assert r <= rel, "%s: rel-L2 %.3e > %.1e" % (name, r, rel)
    scale = float(np.abs(ref64).max()) if ref64.size else 0.0
    worst = float(np.abs(got - ref64).max()) if ref64.size else 0.0
    assert worst <= rel * scale + 1e-30, "%s: max err %.3e > %.1e * %.3e" % (name, worst, rel, scale)


def check_stats(mean_t, rstd_t, mean64, rstd64):
    mean = to_host64(mean_t).reshape(mean64.shape)
    rstd = to_host64(rstd_t).reshape(rstd64.shape)
    rel = np.abs(rstd - rstd64) / rstd64
    assert rel.max() <= 1e-5, "rstd: relative error %.3e > 1e-5" % rel.max()
    std = 1.0 / rstd64
    bound = 1e-5 * np.maximum(np.abs(mean64), std)
    assert np.all(np.abs(mean - mean64) <= bound), "mean: error %.3e beyond 1e-5*max(|mean|, std)" % (
        np.abs(mean - mean64).max())


# ---- the same bounds evaluated on the device, for tensors too large to compare with numpy -------
# The expected values still come from the CPU oracle (float64); only the comparison itself (absolute
# differences, the bounds above, sums of squares) runs as torch operations on the GPU, in float64,
# chunk by chunk.  Per chunk the element-wise bounds use the chunk's own max|ref| (never larger than
# the whole tensor's, so never looser); the relative L2 error is accumulated over all chunks.
class ChunkedCheck:
    def __init__(self, name, dtype):
        self.name, self.dtype = name, dtype
        self.num = 0.0
        self.den = 0.0
        self.rows = 0

    def add(self, got_t, ref64):
        ref = torch.from_numpy(np.ascontiguousarray(ref64)).to(got_t.device)
        got = got_t.reshape(ref.shape).to(torch.float64)
        name = "%s (rows %d...)" % (self.name, self.rows)
        assert bool(torch.isfinite(got).all()), name + ": non-finite values"
        err = (got - ref).abs()
        self.num += float((err * err).sum())
        self.den += float((ref * ref).sum())
        self.rows += ref.shape[0]
        top = float(ref.abs().max())
        if self.dtype == "bf16":
            bad = err > 2e-2 + 2.0 ** -8 * ref.abs()
            assert not bool(bad.any()), "%s: %d elements beyond 2e-2 + 2^-8|ref| (worst %.3e)" % (
                name, int(bad.sum()), float(err.max()))
            rounded = ref.to(torch.bfloat16).to(torch.float64)
            _, expo = torch.frexp(rounded.abs().clamp_min(2.0 ** -126))       # |v| = m 2^e, m in [0.5, 1)
            ulp = torch.ldexp(torch.ones_like(rounded), expo - 8)             # 2^(floor(log2|v|) - 7)
            off = (got - rounded).abs() > ulp * 1.0001 + 1e-5 * top
            assert not bool(off.any()), "%s: %d elements more than one bf16 ulp from the rounded reference" % (
                name, int(off.sum()))
        else:
            assert float(err.max()) <= 1e-5 * top + 1e-30, "%s: max err %.3e > 1e-5 * %.3e" % (
                name, float(err.max()), top)

    def finish(self):
        r = (self.num / self.den) ** 0.5 if self.den > 0 else self.num ** 0.5
        limit = 4e-3 if self.dtype == "bf16" else 1e-5
        assert r <= limit, "%s: rel-L2 %.3e > %.1e over %d rows" % (self.name, r, limit, self.rows)
        return r
