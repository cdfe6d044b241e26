"""GPU test of lnmod_backward_static, the backward entry point that allocates nothing: through the
C ABI, against lnmod_backward (same kernels and plan, so the results must be the same bits), on two
calls in a row, the second with a smaller input; the library must not allocate device memory."""
import pytest
import torch

from paper_2605_17923_amd import lnmod, synth
from parity_util import to_device

pytestmark = pytest.mark.gpu


def _inputs(cfg, dtype, **kw):
    inp = synth.make_inputs(cfg, dtype=dtype, **kw)
    per_token = inp.workload.mod == synth.PER_TOKEN
    B, S, D = inp.B, inp.S, inp.D
    x, dy = to_device(inp.x, dtype).view(B, S, D), to_device(inp.dy, dtype).view(B, S, D)
    scale = to_device(inp.scale, dtype)
    shift = to_device(inp.shift, dtype)
    if per_token:
        scale, shift = scale.view(B, S, D), shift.view(B, S, D)
    return x, dy, shift, scale, per_token


def _both(x, dy, shift, scale, per_token, recompute):
    """(outputs of lnmod_backward, outputs of lnmod_backward_static) on the same inputs."""
    B, S, D = x.shape
    code = lnmod.LNMOD_BF16 if x.dtype == torch.bfloat16 else lnmod.LNMOD_F32
    mod = lnmod.LNMOD_PER_TOKEN if per_token else lnmod.LNMOD_PER_SAMPLE
    st = torch.cuda.current_stream().cuda_stream
    _, mean, rstd = lnmod.forward(x, shift, scale)
    mean, rstd = mean.reshape(-1), rstd.reshape(-1)
    if recompute:
        mean = rstd = None

    def outputs():
        dx = torch.full_like(x, float("nan"))
        if per_token:
            return dx, torch.full_like(x, float("nan")), torch.full_like(x, float("nan"))
        return (dx, torch.full((B, D), float("nan"), device=x.device), torch.full((B, D), float("nan"), device=x.device))

    ref = outputs()
    ws = lnmod.workspace(B, B * S, D, x.device)
    rc = lnmod.lnmod_backward(dy, x, None, scale, B, S, D, 1e-6, st, mean, rstd, ref[0], ref[1], ref[2], ws,
                              ws.numel(), code, mod)
    assert rc == 0, lnmod.lnmod_status_string(rc)
    got = outputs()
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated(), torch.cuda.memory_reserved()
    rc = lnmod.lnmod_backward_static(dy, x, None, scale, B, S, D, 1e-6, st, mean, rstd, got[0], got[1], got[2],
                                     code, mod)
    assert rc == 0, lnmod.lnmod_status_string(rc)
    torch.cuda.synchronize()
    assert (torch.cuda.memory_allocated(), torch.cuda.memory_reserved()) == before
    return ref, got


def _same(ref, got, what):
    for name, a, b in zip(("dx", "dshift", "dscale"), ref, got):
        assert bool(torch.isfinite(b.float()).all()), "%s: %s not written in full" % (what, name)
        assert torch.equal(a, b), "%s: %s differs from lnmod_backward" % (what, name)


def test_two_calls_in_a_row_the_second_smaller():
    # bf16, D = 5120: 2 samples of 3001 rows, then 1 sample of 517 rows of another width; the second
    # call finds the first call's partial sums in the array and must not be disturbed by them
    big = _inputs(2, "bf16", B=2, S=3001)
    small = _inputs(1, "bf16", B=1, S=517, with_dy=True)
    for recompute in (False, True):
        _same(*_both(*big, recompute), "first call, recompute=%s" % recompute)
        _same(*_both(*small, recompute), "second, smaller call, recompute=%s" % recompute)
        _same(*_both(*big, recompute), "third call, large again, recompute=%s" % recompute)


def test_other_layouts_and_types():
    _same(*_both(*_inputs(0, "f32"), False), "fp32 tiny")
    _same(*_both(*_inputs(3, "bf16", B=2, S=301), False), "per token (no workspace)")
    _same(*_both(*_inputs(2, "bf16", B=7, S=129, D=1536), False), "seven samples")


def test_headline_workload_fits_and_too_many_slots_are_refused():
    x, dy, shift, scale, per_token = _inputs(2, "bf16")                  # 75600 x 5120
    _same(*_both(x, dy, shift, scale, per_token, False), "headline workload")
    del x, dy
    # 3000 samples at D = 8192: (clusters + 3000 - 1) * nb slots of 64 KB are more than the array holds
    st = torch.cuda.current_stream().cuda_stream
    A = 0x1000
    assert lnmod.lnmod_backward_static(A, A, None, A, 3000, 40, 8192, 1e-6, st, A, A, A, A, A, lnmod.LNMOD_BF16,
                                       lnmod.LNMOD_PER_SAMPLE) == lnmod.LNMOD_EWORKSPACE
    torch.cuda.synchronize()
