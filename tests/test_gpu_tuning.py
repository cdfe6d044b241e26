"""GPU checks of the tuning interface: results under a launch-shape override still match the
float64 oracle, a combination that was not compiled fails without running anything, and removing
the override restores the table's launch bit for bit."""
import pytest
import torch

from paper_2605_17923_amd import lnmod, synth, tune
from parity_util import to_device
from test_gpu_parity import run_case

pytestmark = pytest.mark.gpu

ALL_FAMILIES = range(lnmod.LNMOD_TUNE_FAMILIES)


@pytest.fixture(autouse=True)
def _no_override_left_behind():
    yield
    for fam in ALL_FAMILIES:
        assert lnmod.lnmod_tuning_set_shape(fam, 0, 0, 0, 0) == 0
    torch.cuda.synchronize()


# shapes that are compiled for bf16 rows of 5120 features (entries of the tables at other widths)
@pytest.mark.parametrize("fwd,bwd,rc", [((4, 3, 1, 2), (5, 2, 2, 1), (8, 2, 2, 1)),
                                         ((6, 3, 1, 1), (6, 2, 1, 3), (4, 3, 2, 4)),
                                         ((5, 2, 1, 3), (8, 2, 1, 2), (4, 3, 1, 1))])
def test_overridden_shapes_match_the_oracle(fwd, bwd, rc):
    assert lnmod.lnmod_tuning_set_shape(lnmod.LNMOD_TUNE_FORWARD, *fwd) == 0
    assert lnmod.lnmod_tuning_set_shape(lnmod.LNMOD_TUNE_BACKWARD, *bwd) == 0
    assert lnmod.lnmod_tuning_set_shape(lnmod.LNMOD_TUNE_BACKWARD_RECOMPUTE, *rc) == 0
    run_case(synth.make_inputs(2, S=2053), label="override %s %s" % (fwd, bwd))
    run_case(synth.make_inputs(2, S=2053), label="override rc %s" % (rc,), recompute=True)
    lengths = (37, 0, 1560, 5, 819, 1, 0, 0, 300, 64, 2, 777, 0)
    run_case(synth.make_inputs(4, lengths=lengths), label="override varlen")


def test_uncompiled_shape_fails_and_reset_restores_the_table_launch():
    inp = synth.make_inputs(2, S=1000)
    assert inp.D == 5120
    x = to_device(inp.x, "bf16").view(1, 1000, inp.D)
    shift, scale = to_device(inp.shift, "bf16"), to_device(inp.scale, "bf16")
    y0, mean0, rstd0 = lnmod.forward(x, shift, scale)
    torch.cuda.synchronize()
    assert lnmod.lnmod_tuning_set_shape(lnmod.LNMOD_TUNE_FORWARD, 7, 2, 1, 1) == 0     # no 7-wave kernel
    with pytest.raises(lnmod.LnmodError):
        lnmod.forward(x, shift, scale)
    assert lnmod.lnmod_tuning_set_shape(lnmod.LNMOD_TUNE_FORWARD, 2, 2, 1, 4) == 0     # 256 of 640 chunks
    with pytest.raises(lnmod.LnmodError):
        lnmod.forward(x, shift, scale)
    assert lnmod.lnmod_tuning_set_shape(lnmod.LNMOD_TUNE_FORWARD, 0, 0, 0, 0) == 0
    y1, mean1, rstd1 = lnmod.forward(x, shift, scale)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1) and torch.equal(mean0, mean1) and torch.equal(rstd0, rstd1)


@pytest.mark.parametrize("family,D", [("forward", 1536), ("backward", 1536), ("backward_recompute", 2048),
                                      ("token_forward", 1024), ("token_backward", 1024),
                                      ("gated_forward", 1536), ("gated_backward", 1536),
                                      ("qknorm_forward", 5120), ("qknorm_backward", 1536)])
def test_sweep_runs_and_contains_the_table_entry(family, D):
    table, before, after, res = tune.sweep(family, D, torch.bfloat16, 8e6, iters=2, warmup=1)
    assert before > 0 and after > 0
    assert len(res) >= 3
    assert all(us > 0 for _, us in res)
    st, again = lnmod.lnmod_tuning_table_shape(tune.FAMILIES[family], D, 0)
    assert st == 0 and again == table


def test_command_line_entry_point(capsys):
    rc = tune.main(["--family", "backward", "--D", "1024", "--bytes", "8e6", "--iters", "2", "--warmup", "1",
                    "--top", "3"])
    assert rc == 0
    out = capsys.readouterr().out
    assert "backward D=1024 bf16: table (1, 2, 2, 3)" in out
    assert out.count(" us") >= 4
