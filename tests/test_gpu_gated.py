"""GPU parity of the gated residual + LayerNorm-Modulate kernels (called through the C ABI)
against the float64 oracle in oracle/gated_oracle.c on the same seeded inputs.

h is a quantised value (one fp32 fused multiply-add rounded to the I/O type), so both sides take
that rounding in the same precision and h is compared bit for bit; y, the statistics and every
gradient are compared with the tolerances of the LayerNorm-Modulate tests.  The GPU backward is fed
the h, mean and rstd the GPU forward produced; the oracle's backward reads the oracle's own h and
recomputes the statistics in float64, so no GPU output enters the expected values."""
import numpy as np
import pytest
import torch

from oracle import gated_oracle as go
from paper_2605_17923_amd import lnmod, synth
from parity_util import check_f32_tensor, check_io_tensor, check_stats, to_device, to_host64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    lnmod.library()
    yield
    torch.cuda.synchronize()


def run_gated(inp, seed, sample_rows=None, label=""):
    w = inp.workload
    dt = w.dtype
    T, D, B = inp.T, inp.D, inp.B
    ex = synth.make_gated_extras(inp, seed)
    print("gated case", label or w.name, "dtype", dt, "T", T, "D", D, "B", B, "varlen", w.varlen, flush=True)
    x, u, dy, dh = (to_device(a, dt) for a in (inp.x, ex.u, inp.dy, ex.dh))
    gate, shift, scale = (to_device(a, dt) for a in (ex.gate, inp.shift, inp.scale))
    cu64 = inp.cu_seqlens.astype(np.int64)
    cu_dev = torch.from_numpy(inp.cu_seqlens.astype(np.int32)).cuda() if w.varlen else None
    if w.varlen:
        h, y, mean, rstd = lnmod.gated_forward(x, u, gate, shift, scale, cu_dev, w.eps)
    else:
        h, y, mean, rstd = lnmod.gated_forward(x.view(B, inp.S, D), u.view(B, inp.S, D), gate, shift, scale,
                                               None, w.eps)
    torch.cuda.synchronize()
    quant = go.QUANT_BF16 if dt == "bf16" else go.QUANT_F32

    rows = np.arange(T) if sample_rows is None else np.asarray(sample_rows, dtype=np.int64)
    rows_t = torch.from_numpy(rows).cuda()
    h64, y64, mean64, rstd64 = go.forward(inp.x, ex.u, ex.gate, inp.shift, inp.scale, w.eps, cu=cu64, quant=quant)
    if dt == "bf16":
        # Every row, on the device (h64 holds bf16 values exactly).  The oracle rounds its float64 sum to
        # float32 and then to bf16, because one fp32 fused multiply-add followed by one store rounding is
        # what "h as stored" means for an fp32 kernel: a reading that follows the arithmetic type of the
        # path, taken because the paper only names the "Gate + Norm" fusion (Sec. 4.4) and defines nothing.
        h_ref = torch.from_numpy(h64).to(torch.bfloat16).cuda()
        differ = int((h.reshape(T, D) != h_ref).sum())
        assert differ == 0, "h: %d elements differ from the rounded reference" % differ
        del h_ref
    else:
        # fp32: the float64 sum of a 48-bit product and a 24-bit addend can itself round
        h_got = to_host64(h.reshape(T, D))
        ulp = np.spacing(np.abs(h64).astype(np.float32)).astype(np.float64)
        assert np.all(np.abs(h_got - h64) <= ulp), "h: beyond one float32 ulp"
        assert np.mean(h_got != h64) < 1e-4
    check_io_tensor("y", y.reshape(T, D)[rows_t], y64[rows], dt)
    check_stats(mean.reshape(T)[rows_t], rstd.reshape(T)[rows_t], mean64[rows], rstd64[rows])

    if w.varlen:
        dx, du, dgate, dsh, dsc = lnmod.gated_backward(dy, dh, h, u, gate, scale, mean, rstd, cu_dev, w.eps)
    else:
        v = lambda t: t.view(B, inp.S, D)
        dx, du, dgate, dsh, dsc = lnmod.gated_backward(v(dy), v(dh), v(h), v(u), gate, scale, mean, rstd,
                                                       None, w.eps)
    torch.cuda.synchronize()
    # the oracle's backward reads the oracle's h (for bf16 the GPU's h was just shown to be the same bits)
    dx64, du64, dg64, dsh64, dsc64 = go.backward(inp.dy, ex.dh, h64, ex.u, ex.gate, inp.scale, w.eps, cu=cu64)
    check_io_tensor("dx", dx.reshape(T, D)[rows_t], dx64[rows], dt)
    check_io_tensor("du", du.reshape(T, D)[rows_t], du64[rows], dt)
    check_f32_tensor("dgate", dgate, dg64)
    check_f32_tensor("dshift", dsh, dsh64)
    check_f32_tensor("dscale", dsc, dsc64)
    if dt != "bf16":
        # fp32: the GPU backward read its own h, up to one float32 ulp from the oracle's on a few elements.
        # Bound what that is worth: the oracle's backward on the GPU's h moves no gradient by more than a
        # tenth of the tolerance above.
        alt = go.backward(inp.dy, ex.dh, h.reshape(T, D).cpu().numpy(), ex.u, ex.gate, inp.scale, w.eps, cu=cu64)
        for name, a_, b_ in zip(("dx", "du", "dgate", "dshift", "dscale"), alt, (dx64, du64, dg64, dsh64, dsc64)):
            check_f32_tensor(name + " (effect of h within one ulp)", a_, b_, rel=1e-6)


def test_gated_tiny_fp32():
    run_gated(synth.make_inputs(0), 2001)


def test_gated_bf16_d5120_outliers():
    run_gated(synth.make_inputs(2, S=1031), 2002)


def test_gated_bf16_d1536_three_samples():
    run_gated(synth.make_inputs(1, B=3, S=701, with_dy=True), 2003)


@pytest.mark.parametrize("D,dtype", [(1528, "bf16"), (200, "bf16"), (8, "bf16"), (8192, "bf16"), (2560, "bf16"),
                                     (3072, "bf16"), (1024, "bf16"), (2048, "bf16"), (3584, "bf16"), (4096, "bf16"),
                                     (4608, "bf16"), (5120, "bf16"), (6144, "bf16"), (7000, "bf16"),
                                     (100, "f32"), (5120, "f32"), (8192, "f32"), (1100, "f32")])
def test_gated_hidden_sizes(D, dtype):
    run_gated(synth.make_inputs(0, B=2, S=67, D=D, dtype=dtype), 2100 + D, label="D=%d %s" % (D, dtype))


def test_gated_varlen_with_empty_segments():
    lengths = (37, 0, 1560, 5, 819, 1, 0, 0, 300, 64, 2, 777, 0)
    run_gated(synth.make_inputs(4, lengths=lengths), 2004)
    run_gated(synth.make_inputs(4, lengths=(0, 0, 129, 0), D=1536), 2005)
    run_gated(synth.make_inputs(4, lengths=(1,), D=512), 2006)


@pytest.mark.parametrize("seed,nseg,maxlen,D", [(1, 300, 40, 1536), (2, 97, 700, 5120), (3, 1000, 6, 512)])
def test_gated_varlen_many_random_segments(seed, nseg, maxlen, D):
    rng = np.random.default_rng(seed)
    lengths = rng.integers(0, maxlen + 1, nseg)
    lengths[rng.random(nseg) < 0.15] = 0
    run_gated(synth.make_inputs(4, lengths=tuple(int(v) for v in lengths), D=D, seed=300 + seed), 2200 + seed,
              label="random segments nseg=%d maxlen=%d D=%d" % (nseg, maxlen, D))


def test_gated_many_samples():
    run_gated(synth.make_inputs(2, B=200, S=97, D=1024), 2007, label="B=200 S=97 D=1024")


def test_gated_zero_gate_matches_plain_forward():
    # gate = 0: h must equal x bit for bit; y, mean, rstd must agree with lnmod_forward's up to the
    # order of the fp32 row sums (the two kernels may split a row over different numbers of waves)
    inp = synth.make_inputs(2, S=515)
    x = to_device(inp.x, "bf16").view(1, 515, 5120)
    u = to_device(synth.make_gated_extras(inp, 5).u, "bf16").view(1, 515, 5120)
    shift, scale = to_device(inp.shift, "bf16"), to_device(inp.scale, "bf16")
    h, y, mean, rstd = lnmod.gated_forward(x, u, torch.zeros_like(shift), shift, scale)
    y2, mean2, rstd2 = lnmod.forward(x, shift, scale)
    torch.cuda.synchronize()
    assert torch.equal(h, x)
    yd, y2d = y.double(), y2.double()
    assert float(((yd - y2d).abs() / (y2d.abs() + 1e-3)).max()) <= 2.0 ** -7       # at most one bf16 rounding apart
    assert float((yd != y2d).double().mean()) < 0.02
    assert torch.allclose(mean, mean2.reshape(-1), rtol=1e-6, atol=1e-6)
    assert torch.allclose(rstd, rstd2.reshape(-1), rtol=1e-6, atol=0)


def test_gated_results_repeat_bit_for_bit():
    inp = synth.make_inputs(4, lengths=(700, 0, 1300, 41), D=5120)
    ex = synth.make_gated_extras(inp, 9)
    dev = {k: to_device(v, "bf16") for k, v in dict(x=inp.x, u=ex.u, dy=inp.dy, dh=ex.dh, gate=ex.gate,
                                                    shift=inp.shift, scale=inp.scale).items()}
    cu = torch.from_numpy(inp.cu_seqlens.astype(np.int32)).cuda()
    outs = []
    for _ in range(2):
        h, y, mean, rstd = lnmod.gated_forward(dev["x"], dev["u"], dev["gate"], dev["shift"], dev["scale"], cu)
        outs.append((h, y, mean, rstd) + lnmod.gated_backward(dev["dy"], dev["dh"], h, dev["u"], dev["gate"],
                                                              dev["scale"], mean, rstd, cu))
    torch.cuda.synchronize()
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def _sample_rows(T, cu, n=1200, seed=11):
    rng = np.random.default_rng(seed)
    rows = set(rng.integers(0, T, n).tolist())
    rows.update([0, 1, 2, 3, T - 1, T - 2, T - 3, T - 4])
    for c in np.asarray(cu, dtype=np.int64):
        for d in (-2, -1, 0, 1):
            if 0 <= c + d < T:
                rows.add(int(c + d))
    return np.array(sorted(rows), dtype=np.int64)


def test_gated_config2_full_size():
    inp = synth.make_inputs(2)
    run_gated(inp, 2008, sample_rows=_sample_rows(inp.T, inp.cu_seqlens))


def test_gated_tensors_beyond_4_gib():
    # 450 000 tokens x 5120 bf16 = 4.6 GB per tensor (byte offsets pass 2^32); inputs drawn on the device,
    # the oracle checks sampled rows of h, y, dx and du, most of them beyond the 4 GiB line
    T, D = 450_000, 5120
    g = torch.Generator(device="cuda")
    g.manual_seed(777)

    def big(std, mean=0.0):
        t = torch.empty(T, D, device="cuda", dtype=torch.bfloat16)
        for lo in range(0, T, 50_000):
            hi = min(T, lo + 50_000)
            t[lo:hi] = (torch.randn(hi - lo, D, generator=g, device="cuda") * std + mean).to(torch.bfloat16)
        return t

    x, u, dy, dh = big(2.0, 0.5), big(1.0), big(1.0), big(1.0)
    small = lambda s: (s * torch.randn(1, D, generator=g, device="cuda")).to(torch.bfloat16)
    gate, shift, scale = small(0.3), small(0.1), small(0.1)
    v = lambda t: t.view(1, T, D)
    h, y, mean, rstd = lnmod.gated_forward(v(x), v(u), gate, shift, scale, None, 1e-6)
    dx, du, dgate, dsh, dsc = lnmod.gated_backward(v(dy), v(dh), h, v(u), gate, scale, mean, rstd, None, 1e-6)
    torch.cuda.synchronize()
    first_beyond = (1 << 32) // (D * 2) + 1
    rng = np.random.default_rng(6)
    rows = np.unique(np.concatenate([rng.integers(0, T, 100), rng.integers(first_beyond, T, 500),
                                     [0, first_beyond - 1, first_beyond, T - 1]]))
    rt = torch.from_numpy(rows).cuda()
    host = lambda t: t.reshape(-1, D)[rt].float().cpu().numpy()
    row = lambda t: t.float().cpu().numpy()
    h64, y64, mean64, rstd64 = go.forward(host(x), host(u), row(gate), row(shift), row(scale), 1e-6, B=1,
                                          S=rows.size, quant=go.QUANT_BF16)
    assert np.array_equal(to_host64(h.reshape(T, D)[rt]), h64)
    check_io_tensor("y", y.reshape(T, D)[rt], y64, "bf16")
    check_stats(mean.reshape(T)[rt], rstd.reshape(T)[rt], mean64, rstd64)
    # dx and du of a row need only that row (and the modulation rows)
    dx64, du64, _, _, _ = go.backward(host(dy), host(dh), host(h), host(u), row(gate), row(scale), 1e-6, B=1,
                                      S=rows.size)
    check_io_tensor("dx", dx.reshape(T, D)[rt], dx64, "bf16")
    check_io_tensor("du", du.reshape(T, D)[rt], du64, "bf16")
    assert bool(torch.isfinite(dgate).all()) and bool(torch.isfinite(dsh).all()) and bool(torch.isfinite(dsc).all())


def test_gated_every_supported_hidden_size_launches():
    # every D the header promises must map to an instantiated kernel in both gated entry points; 3
    # rows are checked against a float64 torch expression of the definition (not the oracle: 3000
    # sizes, tiny rows), so a launch shape that does not cover its row shows here
    st = torch.cuda.current_stream().cuda_stream
    g = torch.Generator(device="cuda")
    g.manual_seed(11)
    S = 3
    for dtype, code, step, tol in ((torch.bfloat16, lnmod.LNMOD_BF16, 8, 3e-2), (torch.float32, lnmod.LNMOD_F32, 4, 2e-4)):
        bad = []
        for D in range(8, 8193, step):
            big = lambda: torch.randn(S, D, generator=g, device="cuda").to(dtype)      # noqa: E731
            small = lambda: (0.1 * torch.randn(1, D, generator=g, device="cuda")).to(dtype)   # noqa: E731
            x, u, dy, dh = big(), big(), big(), big()
            gate, sh, sc = small(), small(), small()
            h, y, dx, du = (torch.empty_like(x) for _ in range(4))
            mean, rstd = torch.empty(S, device="cuda"), torch.empty(S, device="cuda")
            dg, dsh, dsc = (torch.empty(1, D, device="cuda") for _ in range(3))
            ws = lnmod.gated_workspace(1, S, D, "cuda")
            rc1 = lnmod.lnmod_gated_forward(x, u, gate, sh, sc, None, 1, S, D, 1e-6, st, h, y, mean, rstd, code)
            rc2 = lnmod.lnmod_gated_backward(dy, dh, h, u, gate, sc, None, 1, S, D, 1e-6, st, mean, rstd, dx, du, dg,
                                             dsh, dsc, ws, ws.numel(), code)
            if rc1 != 0 or rc2 != 0:
                bad.append((D, rc1, rc2))
                continue
            xd, ud, dyd, dhd, gd, scd, shd = (t.double() for t in (x, u, dy, dh, gate, sc, sh))
            want_h = xd + gd * ud
            assert float((h.double() - want_h).abs().max()) <= tol * float(want_h.abs().max() + 1), D
            hd = h.double()                                  # the stored h is what is normalised
            mu = hd.mean(1, keepdim=True)
            r = 1.0 / torch.sqrt(((hd - mu) ** 2).mean(1, keepdim=True) + 1e-6)
            xh = (hd - mu) * r
            gg = dyd * (1 + scd)
            want_dx = dhd + r * (gg - gg.mean(1, keepdim=True) - xh * (gg * xh).mean(1, keepdim=True))
            assert float((y.double() - (xh * (1 + scd) + shd)).abs().max()) <= tol * 4, D
            assert float((dx.double() - want_dx).abs().max()) <= tol * float(want_dx.abs().max() + 1), D
            # du and dgate are formed from the unrounded dx
            assert float((du.double() - gd * want_dx).abs().max()) <= tol * float(want_dx.abs().max() + 1), D
            want_dg = (want_dx * ud).sum(0, keepdim=True)
            assert float((dg.double() - want_dg).abs().max()) <= tol * float(want_dg.abs().max() + 1), D
            assert float((dsh.double() - dyd.sum(0, keepdim=True)).abs().max()) <= 1e-4, D
            assert float((dsc.double() - (dyd * xh).sum(0, keepdim=True)).abs().max()) <= 1e-3, D
        torch.cuda.synchronize()
        assert not bad, "launch failed for %d sizes, first %r" % (len(bad), bad[:5])
