"""The torch.autograd wrappers must be pure wiring: outputs and gradients identical, bit for bit, to
what the direct binding calls give on the same inputs (those calls are what the parity tests compare
with the oracle), parameter gradients cast once to the parameters' dtype; one case is also checked
against the float64 oracle end to end."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_17923_amd import functional as F
from paper_2605_17923_amd import lnmod, synth
from parity_util import check_io_tensor, to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    lnmod.library()
    yield
    torch.cuda.synchronize()


def _leaf(a, dt):
    return to_device(a, dt).requires_grad_(True)


@pytest.mark.parametrize("cfg,kw,save_stats", [(0, {}, True), (2, dict(S=777), True), (2, dict(S=777), False),
                                               (3, dict(B=2, S=131), True),
                                               (4, dict(lengths=[0, 301, 1, 0, 977, 64]), True),
                                               (4, dict(lengths=[5, 0, 40]), False)])
def test_ln_modulate_matches_direct_calls(cfg, kw, save_stats):
    inp = synth.make_inputs(cfg, **kw)
    w = inp.workload
    dt, B, D = w.dtype, inp.B, inp.D
    per_token = w.mod == synth.PER_TOKEN
    shape = (inp.T, D) if w.varlen else (B, inp.S, D)
    mshape = shape if per_token else (B, D)
    x = _leaf(inp.x.reshape(shape), dt)
    shift, scale = _leaf(inp.shift.reshape(mshape), dt), _leaf(inp.scale.reshape(mshape), dt)
    dy = to_device(inp.dy.reshape(shape), dt)
    cu = torch.from_numpy(inp.cu_seqlens.astype(np.int32)).cuda() if w.varlen else None
    y = F.ln_modulate(x, shift, scale, eps=w.eps, cu_seqlens=cu, save_stats=save_stats)
    y.backward(dy)
    torch.cuda.synchronize()
    xd, shd, scd = x.detach(), shift.detach(), scale.detach()
    if w.varlen:
        y0, mean, rstd = lnmod.forward_varlen(xd, shd, scd, cu, w.eps)
        dx0, dsh0, dsc0 = lnmod.backward_varlen(dy, xd, scd, cu, mean if save_stats else None,
                                                rstd if save_stats else None, w.eps)
    else:
        y0, mean, rstd = lnmod.forward(xd, shd, scd, w.eps)
        dx0, dsh0, dsc0 = lnmod.backward(dy, xd, scd, mean if save_stats else None,
                                         rstd if save_stats else None, w.eps)
    torch.cuda.synchronize()
    assert torch.equal(y.detach(), y0)
    assert torch.equal(x.grad, dx0)
    assert shift.grad.dtype == shift.dtype and scale.grad.dtype == scale.dtype
    assert torch.equal(shift.grad, dsh0.to(shift.dtype).reshape(mshape))
    assert torch.equal(scale.grad, dsc0.to(scale.dtype).reshape(mshape))


def test_ln_modulate_gradients_against_the_oracle():
    inp = synth.make_inputs(2, S=513)
    w = inp.workload
    x = _leaf(inp.x.reshape(1, -1, inp.D), "bf16")
    shift, scale = _leaf(inp.shift, "bf16"), _leaf(inp.scale, "bf16")
    y = F.ln_modulate(x, shift, scale, eps=w.eps)
    y.backward(to_device(inp.dy.reshape(1, -1, inp.D), "bf16"))
    torch.cuda.synchronize()
    y64, _, _ = oracle.forward(inp.x, inp.shift, inp.scale, w.eps, cu=inp.cu_seqlens.astype(np.int64))
    dx64, dsh64, dsc64 = oracle.backward(inp.dy, inp.x, inp.scale, w.eps, cu=inp.cu_seqlens.astype(np.int64))
    check_io_tensor("y", y.detach(), y64, "bf16")
    check_io_tensor("x.grad", x.grad, dx64, "bf16")
    check_io_tensor("shift.grad", shift.grad, dsh64, "bf16")        # bf16 parameters: one rounding of the sum
    check_io_tensor("scale.grad", scale.grad, dsc64, "bf16")


@pytest.mark.parametrize("varlen", [False, True])
def test_gated_ln_modulate_matches_direct_calls(varlen):
    inp = synth.make_inputs(4, lengths=[0, 211, 3, 500]) if varlen else synth.make_inputs(2, B=2, S=333)
    w = inp.workload
    dt, B, D = w.dtype, inp.B, inp.D
    ex = synth.make_gated_extras(inp, 77)
    shape = (inp.T, D) if varlen else (B, inp.S, D)
    x, u = _leaf(inp.x.reshape(shape), dt), _leaf(ex.u.reshape(shape), dt)
    gate, shift, scale = _leaf(ex.gate, dt), _leaf(inp.shift, dt), _leaf(inp.scale, dt)
    dy, dh = to_device(inp.dy.reshape(shape), dt), to_device(ex.dh.reshape(shape), dt)
    cu = torch.from_numpy(inp.cu_seqlens.astype(np.int32)).cuda() if varlen else None
    h, y = F.gated_ln_modulate(x, u, gate, shift, scale, eps=w.eps, cu_seqlens=cu)
    torch.autograd.backward([h, y], [dh, dy])
    torch.cuda.synchronize()
    d = lambda t: t.detach()
    h0, y0, mean, rstd = lnmod.gated_forward(d(x), d(u), d(gate), d(shift), d(scale), cu, w.eps)
    dx0, du0, dg0, dsh0, dsc0 = lnmod.gated_backward(dy, dh, h0, d(u), d(gate), d(scale), mean, rstd, cu, w.eps)
    torch.cuda.synchronize()
    assert torch.equal(d(h), h0) and torch.equal(d(y), y0)
    assert torch.equal(x.grad, dx0) and torch.equal(u.grad, du0)
    assert torch.equal(gate.grad, dg0.to(gate.dtype))
    assert torch.equal(shift.grad, dsh0.to(shift.dtype)) and torch.equal(scale.grad, dsc0.to(scale.dtype))


@pytest.mark.parametrize("N,D,dtype", [(1000, 5120, "bf16"), (4096, 128, "bf16"), (300, 1536, "f32")])
def test_qk_norm_matches_direct_calls(N, D, dtype):
    qi = synth.make_qknorm_inputs(N, D, dtype, 91)
    q, k = _leaf(qi.q, dtype), _leaf(qi.k, dtype)
    wq, wk = _leaf(qi.wq, dtype), _leaf(qi.wk, dtype)
    dqo, dko = to_device(qi.dq_out, dtype), to_device(qi.dk_out, dtype)
    qn, kn = F.qk_norm(q, k, wq, wk, eps=1e-6)
    torch.autograd.backward([qn, kn], [dqo, dko])
    torch.cuda.synchronize()
    d = lambda t: t.detach()
    qn0, kn0, rq, rk = lnmod.qknorm_forward(d(q), d(k), d(wq), d(wk), 1e-6)
    dq0, dk0, dwq0, dwk0 = lnmod.qknorm_backward(dqo, dko, d(q), d(k), d(wq), d(wk), rq, rk, 1e-6)
    torch.cuda.synchronize()
    assert torch.equal(d(qn), qn0) and torch.equal(d(kn), kn0)
    assert torch.equal(q.grad, dq0) and torch.equal(k.grad, dk0)
    assert torch.equal(wq.grad, dwq0.to(wq.dtype)) and torch.equal(wk.grad, dwk0.to(wk.dtype))


def test_non_contiguous_input_is_refused():
    x = torch.randn(2, 8, 64, device="cuda").transpose(0, 1)
    s = torch.zeros(8, 64, device="cuda")
    with pytest.raises(ValueError):
        F.ln_modulate(x, s, s)
