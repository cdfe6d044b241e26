"""GPU parity of the fused Q-Norm + K-Norm kernels (called through the C ABI) against the float64
oracle in oracle/qknorm_oracle.c on the same seeded inputs, with the tolerances of the
LayerNorm-Modulate tests (bf16 tensors: rel-L2 4e-3 and one bf16 rounding; fp32 tensors and the
float32 weight gradients: 1e-5; rstd: 1e-5 relative)."""
import numpy as np
import pytest
import torch

from oracle import qknorm_oracle as qo
from paper_2605_17923_amd import lnmod, synth
from parity_util import check_f32_tensor, check_io_tensor, to_device, to_host64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    lnmod.library()
    yield
    torch.cuda.synchronize()


def run_qk(inp, sample_rows=None, label=""):
    dt = inp.dtype
    N, D = inp.q.shape
    print("qknorm case", label, "dtype", dt, "N", N, "D", D, flush=True)
    q, k, wq, wk, dqo, dko = (to_device(a, dt) for a in (inp.q, inp.k, inp.wq, inp.wk, inp.dq_out, inp.dk_out))
    q_out, k_out, rq, rk = lnmod.qknorm_forward(q, k, wq, wk, inp.eps)
    dq, dk, dwq, dwk = lnmod.qknorm_backward(dqo, dko, q, k, wq, wk, rq, rk, inp.eps)
    torch.cuda.synchronize()
    rows = np.arange(N) if sample_rows is None else np.asarray(sample_rows, dtype=np.int64)
    rows_t = torch.from_numpy(rows).cuda()
    for name, x, w, dy, y_g, r_g, dx_g, dw_g in (("q", inp.q, inp.wq, inp.dq_out, q_out, rq, dq, dwq),
                                                 ("k", inp.k, inp.wk, inp.dk_out, k_out, rk, dk, dwk)):
        y64, r64 = qo.forward_one(x[rows], w, inp.eps)              # rows are independent in the forward
        check_io_tensor(name + "_out", y_g[rows_t], y64, dt)
        rel = np.abs(to_host64(r_g[rows_t]) - r64) / r64
        assert rel.max() <= 1e-5, "rstd_%s: relative error %.3e" % (name, rel.max())
        dx64, dw64 = qo.backward_one(dy, x, w, inp.eps)
        check_io_tensor("d" + name, dx_g[rows_t], dx64[rows], dt)
        check_f32_tensor("dw" + name, dw_g, dw64)


def test_qknorm_bf16_d5120():
    run_qk(synth.make_qknorm_inputs(1031, 5120, "bf16", 3001))


def test_qknorm_bf16_d1536():
    run_qk(synth.make_qknorm_inputs(2311, 1536, "bf16", 3002))


def test_qknorm_fp32_d1536():
    run_qk(synth.make_qknorm_inputs(512, 1536, "f32", 3003))


@pytest.mark.parametrize("D,dtype", [(8, "bf16"), (128, "bf16"), (200, "bf16"), (1528, "bf16"), (2560, "bf16"),
                                     (3072, "bf16"), (8192, "bf16"), (100, "f32"),
                                     (128, "f32"), (1100, "f32"), (5120, "f32"), (8192, "f32")])
def test_qknorm_hidden_sizes(D, dtype):
    run_qk(synth.make_qknorm_inputs(131, D, dtype, 3100 + D), label="D=%d %s" % (D, dtype))


@pytest.mark.parametrize("N", [1, 2, 3, 255, 257, 513])
def test_qknorm_row_counts(N):
    run_qk(synth.make_qknorm_inputs(N, 1024, "bf16", 3200 + N), label="N=%d" % N)


@pytest.mark.parametrize("N", [1, 3, 4, 5, 31, 32, 33, 127, 4099])
@pytest.mark.parametrize("D,dtype", [(128, "bf16"), (256, "bf16"), (64, "bf16"), (64, "f32"), (72, "bf16")])
def test_qknorm_short_rows(N, D, dtype):
    # rows of at most 32 chunks take the 16-lanes-per-row kernels: ragged piece and group tails
    run_qk(synth.make_qknorm_inputs(N, D, dtype, 3300 + N + D), label="short N=%d D=%d %s" % (N, D, dtype))


def test_qknorm_per_head_view():
    # one head's width as the normalised dimension: [tokens*heads, 128]
    run_qk(synth.make_qknorm_inputs(300 * 40, 128, "bf16", 3004), label="per head")


def test_qknorm_zero_rows_and_zero_inputs():
    inp = synth.make_qknorm_inputs(64, 512, "bf16", 3005)
    inp.q[3, :] = 0.0                       # rstd = 1/sqrt(eps), y = 0, dx = rstd * dy * w
    inp.k[:] = 0.0
    run_qk(inp, label="zero rows")


def test_qknorm_empty_and_repeatable():
    D = 512
    z = torch.empty(0, D, dtype=torch.bfloat16, device="cuda")
    w = torch.ones(D, dtype=torch.bfloat16, device="cuda")
    q_out, k_out, rq, rk = lnmod.qknorm_forward(z, z, w, w)
    dq, dk, dwq, dwk = lnmod.qknorm_backward(z, z, z, z, w, w, rq, rk)
    torch.cuda.synchronize()
    assert q_out.shape == (0, D) and torch.all(dwq == 0) and torch.all(dwk == 0)
    inp = synth.make_qknorm_inputs(777, 5120, "bf16", 3006)
    dev = [to_device(a, "bf16") for a in (inp.q, inp.k, inp.wq, inp.wk, inp.dq_out, inp.dk_out)]
    outs = []
    for _ in range(2):
        f = lnmod.qknorm_forward(*dev[:4])
        outs.append(f + lnmod.qknorm_backward(dev[4], dev[5], dev[0], dev[1], dev[2], dev[3], f[2], f[3]))
    torch.cuda.synchronize()
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_qknorm_full_size():
    inp = synth.make_qknorm_inputs(75600, 5120, "bf16", 3007)
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([rng.integers(0, 75600, 1000), [0, 1, 2, 75597, 75598, 75599]]))
    run_qk(inp, sample_rows=rows, label="full size")


def test_qknorm_tensors_beyond_4_gib():
    # 450 000 rows x 5120 bf16 = 4.6 GB per tensor (byte offsets pass 2^32); inputs drawn on the device,
    # the oracle checks sampled rows of both outputs and both input gradients beyond the 4 GiB line
    N, D = 450_000, 5120
    g = torch.Generator(device="cuda")
    g.manual_seed(778)

    def big(std, mean=0.0):
        t = torch.empty(N, D, device="cuda", dtype=torch.bfloat16)
        for lo in range(0, N, 50_000):
            hi = min(N, lo + 50_000)
            t[lo:hi] = (torch.randn(hi - lo, D, generator=g, device="cuda") * std + mean).to(torch.bfloat16)
        return t

    q, k, dqo, dko = big(1.0), big(2.0, 0.2), big(1.0), big(1.0)
    wq = (1 + 0.1 * torch.randn(D, generator=g, device="cuda")).to(torch.bfloat16)
    wk = (1 + 0.1 * torch.randn(D, generator=g, device="cuda")).to(torch.bfloat16)
    q_out, k_out, rq, rk = lnmod.qknorm_forward(q, k, wq, wk, 1e-6)
    dq, dk, dwq, dwk = lnmod.qknorm_backward(dqo, dko, q, k, wq, wk, rq, rk, 1e-6)
    torch.cuda.synchronize()
    first_beyond = (1 << 32) // (D * 2) + 1
    rng = np.random.default_rng(8)
    rows = np.unique(np.concatenate([rng.integers(0, N, 100), rng.integers(first_beyond, N, 500),
                                     [0, first_beyond - 1, first_beyond, N - 1]]))
    rt = torch.from_numpy(rows).cuda()
    host = lambda t: t[rt].float().cpu().numpy()
    vec = lambda t: t.float().cpu().numpy()
    for name, x_, w_, out_, dyo_, dx_ in (("q", q, wq, q_out, dqo, dq), ("k", k, wk, k_out, dko, dk)):
        y64, _ = qo.forward_one(host(x_), vec(w_), 1e-6)
        check_io_tensor(name + "_out", out_[rt], y64, "bf16")
        dx64, _ = qo.backward_one(host(dyo_), host(x_), vec(w_), 1e-6)    # dx of a row needs only that row
        check_io_tensor("d" + name, dx_[rt], dx64, "bf16")
    assert bool(torch.isfinite(dwq).all()) and bool(torch.isfinite(dwk).all())


def test_qknorm_every_supported_hidden_size_launches():
    # every D the header promises must map to an instantiated kernel (short rows, wide rows, every
    # launch-shape override); 5 rows are checked against a float64 torch expression of the definition
    st = torch.cuda.current_stream().cuda_stream
    g = torch.Generator(device="cuda")
    g.manual_seed(13)
    N = 5
    for dtype, code, step, tol in ((torch.bfloat16, lnmod.LNMOD_BF16, 8, 3e-2), (torch.float32, lnmod.LNMOD_F32, 4, 2e-4)):
        bad = []
        for D in range(8, 8193, step):
            big = lambda: torch.randn(N, D, generator=g, device="cuda").to(dtype)      # noqa: E731
            wgt = lambda: (1.0 + 0.1 * torch.randn(D, generator=g, device="cuda")).to(dtype)   # noqa: E731
            q, k, dqo, dko = big(), big(), big(), big()
            wq, wk = wgt(), wgt()
            qo, ko, dq, dk = (torch.empty_like(q) for _ in range(4))
            rq, rk = torch.empty(N, device="cuda"), torch.empty(N, device="cuda")
            dwq, dwk = torch.empty(D, device="cuda"), torch.empty(D, device="cuda")
            nbytes = lnmod.lnmod_qknorm_backward_workspace_bytes(N, D)
            ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
            rc1 = lnmod.lnmod_qknorm_forward(q, k, wq, wk, N, D, 1e-6, st, qo, ko, rq, rk, code)
            rc2 = lnmod.lnmod_qknorm_backward(dqo, dko, q, k, wq, wk, N, D, 1e-6, st, rq, rk, dq, dk, dwq, dwk, ws,
                                              ws.numel(), code)
            if rc1 != 0 or rc2 != 0:
                bad.append((D, rc1, rc2))
                continue
            for x, w, dy, y, dx, dw in ((q, wq, dqo, qo, dq, dwq), (k, wk, dko, ko, dk, dwk)):
                xd, wd, dyd = x.double(), w.double(), dy.double()
                r = 1.0 / torch.sqrt((xd * xd).mean(1, keepdim=True) + 1e-6)
                xh = xd * r
                gg = dyd * wd
                want_dx = r * (gg - xh * (gg * xh).mean(1, keepdim=True))
                assert float((y.double() - xh * wd).abs().max()) <= tol * 4, D
                assert float((dx.double() - want_dx).abs().max()) <= tol * float(want_dx.abs().max() + 1), D
                assert float((dw.double() - (dyd * xh).sum(0)).abs().max()) <= 1e-3, D
        torch.cuda.synchronize()
        assert not bad, "launch failed for %d sizes, first %r" % (len(bad), bad[:5])
