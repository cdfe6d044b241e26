"""GPU checks of the measurement library's shaped calls (include/lnmod_tools.h): results under a
given launch shape still match the float64 oracle, a combination that was not compiled fails
without running anything, and shape = NULL is the operator library's launch bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_17923_amd import lnmod, lnmod_tools, synth
from parity_util import check_f32_tensor, check_io_tensor, check_stats, to_device

pytestmark = pytest.mark.gpu


def shaped_forward(shape, x, shift, scale, cu, n, s_or_t, D, mod=0):
    T = x.shape[0]
    y = torch.empty_like(x)
    mean = torch.empty(T, dtype=torch.float32, device=x.device)
    rstd = torch.empty(T, dtype=torch.float32, device=x.device)
    st = lnmod_tools.lnmod_forward_shaped(shape, x, shift, scale, cu, n, s_or_t, D, 1e-6,
                                          torch.cuda.current_stream().cuda_stream, y, mean, rstd, lnmod.LNMOD_BF16, mod)
    return st, y, mean, rstd


def shaped_backward(shape, dy, x, scale, cu, n, s_or_t, D, mean, rstd):
    T = x.shape[0]
    dx = torch.empty_like(x)
    dsh = torch.empty(n, D, dtype=torch.float32, device=x.device)
    dsc = torch.empty(n, D, dtype=torch.float32, device=x.device)
    need = lnmod_tools.lnmod_backward_workspace_bytes_shaped(shape, n, T, D, 0)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    st = lnmod_tools.lnmod_backward_shaped(shape, dy, x, scale, cu, n, s_or_t, D, 1e-6,
                                           torch.cuda.current_stream().cuda_stream, mean, rstd, dx, dsh, dsc, ws,
                                           ws.numel(), lnmod.LNMOD_BF16, 0)
    return st, dx, dsh, dsc


def run_shaped(inp, fwd, bwd, rc, label):
    """Forward with shape `fwd`, backward with saved statistics (`bwd`) and without (`rc`)."""
    print("shaped case", label, fwd, bwd, rc, flush=True)
    w = inp.workload
    T, D = inp.T, inp.D
    x, dy = to_device(inp.x, "bf16"), to_device(inp.dy, "bf16")
    shift, scale = to_device(inp.shift, "bf16"), to_device(inp.scale, "bf16")
    cu64 = inp.cu_seqlens.astype(np.int64)
    cu = torch.from_numpy(inp.cu_seqlens.astype(np.int32)).cuda() if w.varlen else None
    n, s_or_t = (inp.B, T) if w.varlen else (inp.B, inp.S)
    st, y, mean, rstd = shaped_forward(fwd, x, shift, scale, cu, n, s_or_t, D)
    assert st == 0, lnmod.lnmod_status_string(st)
    torch.cuda.synchronize()
    y64, mean64, rstd64 = oracle.forward(inp.x, inp.shift, inp.scale, w.eps, cu=cu64)
    check_io_tensor("y", y, y64, "bf16")
    check_stats(mean, rstd, mean64, rstd64)
    dx64, dsh64, dsc64 = oracle.backward(inp.dy, inp.x, inp.scale, w.eps, cu=cu64)
    for shape, stats in ((bwd, (mean, rstd)), (rc, (None, None))):
        st, dx, dsh, dsc = shaped_backward(shape, dy, x, scale, cu, n, s_or_t, D, *stats)
        assert st == 0, lnmod.lnmod_status_string(st)
        torch.cuda.synchronize()
        check_io_tensor("dx", dx, dx64, "bf16")
        check_f32_tensor("dshift", dsh, dsh64)
        check_f32_tensor("dscale", dsc, dsc64)


# shapes that are compiled for bf16 rows of 5120 features (entries of the tables at other widths)
@pytest.mark.parametrize("fwd,bwd,rc", [((4, 3, 1, 2), (5, 2, 2, 1), (8, 2, 2, 1)),
                                         ((6, 3, 1, 1), (6, 2, 1, 3), (4, 3, 2, 4)),
                                         ((5, 2, 1, 3), (8, 2, 1, 2), (4, 3, 1, 1))])
def test_given_shapes_match_the_oracle(fwd, bwd, rc):
    run_shaped(synth.make_inputs(2, S=2053), fwd, bwd, rc, "one sample")
    lengths = (37, 0, 1560, 5, 819, 1, 0, 0, 300, 64, 2, 777, 0)
    run_shaped(synth.make_inputs(4, lengths=lengths), fwd, bwd, rc, "varlen")


@pytest.mark.parametrize("clusters,interleave", [(8, 1), (8, 0), (3, 1), (2, 0), (64, 1)])
def test_given_cluster_counts_and_block_interleaving_match_the_oracle(clusters, interleave):
    # clusters of blocks with their own share of the rows, either made of consecutive blocks or of every
    # clusters-th block (all of one cluster on one XCD when there are 8): same results, other slots
    fwd, bwd, rc = (5, 2, 2, 1, clusters, interleave), (4, 3, 2, 1, clusters, interleave), (4, 3, 1, 2, clusters, interleave)
    run_shaped(synth.make_inputs(2, S=2053), fwd, bwd, rc, "one sample, %d clusters" % clusters)
    lengths = (37, 0, 1560, 5, 819, 1, 0, 0, 300, 64, 2, 777, 0)
    run_shaped(synth.make_inputs(4, lengths=lengths), fwd, bwd, rc, "varlen, %d clusters" % clusters)


@pytest.mark.parametrize("clusters", [0, 1, 2, 5, 64])
def test_one_loop_over_all_rows_gives_the_forward_of_one_loop_per_segment_bit_for_bit(clusters):
    # shape[6] = 1: the block's rows are taken whatever segment they fall in and the modulation registers
    # are reloaded where the segment changes; = 2: one loop per segment.  Same shape, same row arithmetic.
    lengths = (37, 0, 1560, 5, 819, 1, 0, 0, 300, 64, 2, 777, 0, 1, 1, 1, 2, 0, 3, 2049, 0)
    for D, base in ((5120, (5, 2, 2, 1)), (5120, (4, 3, 1, 2)), (1536, (1, 3, 2, 4)), (1528, (1, 3, 2, 4))):
        inp = synth.make_inputs(4, lengths=lengths, D=D, seed=11)
        print("flat against per-segment", D, base, clusters, flush=True)
        x = to_device(inp.x, "bf16")
        shift, scale = to_device(inp.shift, "bf16"), to_device(inp.scale, "bf16")
        cu = torch.from_numpy(inp.cu_seqlens.astype(np.int32)).cuda()
        outs = []
        for flat in (1, 2):
            st, y, mean, rstd = shaped_forward(base + (clusters, 1, flat), x, shift, scale, cu, inp.B, inp.T, D)
            assert st == 0, lnmod.lnmod_status_string(st)
            torch.cuda.synchronize()
            outs.append((y, mean, rstd))
        for a, b in zip(*outs):
            assert torch.equal(a, b)
        y64, mean64, rstd64 = oracle.forward(inp.x, inp.shift, inp.scale, inp.workload.eps,
                                             cu=inp.cu_seqlens.astype(np.int64))
        check_io_tensor("y", outs[0][0], y64, "bf16")
        check_stats(outs[0][1], outs[0][2], mean64, rstd64)


def test_one_loop_over_all_rows_on_random_segment_tables():
    # random tables with many empty and one-row segments, token counts below and above the grid, cluster
    # regions that end inside, at and between segment boundaries: the two forward loops agree bit for bit
    rng = np.random.default_rng(2024)
    D = 1024
    for case in range(24):
        nseg = int(rng.integers(2, 70))
        kind = case % 4
        if kind == 0:
            lengths = rng.integers(0, 4, size=nseg)                   # fewer rows than blocks
        elif kind == 1:
            lengths = rng.integers(0, 400, size=nseg) * (rng.random(nseg) < 0.5)
        elif kind == 2:
            lengths = np.full(nseg, 64)                               # boundaries on the step grid
        else:
            lengths = rng.integers(1, 3000, size=nseg) * (rng.random(nseg) < 0.3) + (rng.random(nseg) < 0.2)
        lengths = [int(v) for v in lengths]
        if sum(lengths) == 0:
            lengths[nseg // 2] = 1
        clusters = int(rng.choice([0, 1, 2, 3, 8, 32, 256]))
        base = [(1, 2, 2, 4), (2, 2, 1, 4), (1, 2, 1, 8)][case % 3]
        print("random table", case, "nseg", nseg, "T", sum(lengths), "clusters", clusters, base, flush=True)
        inp = synth.make_inputs(4, lengths=lengths, D=D, seed=100 + case, with_dy=False)
        x = to_device(inp.x, "bf16")
        shift, scale = to_device(inp.shift, "bf16"), to_device(inp.scale, "bf16")
        cu = torch.from_numpy(inp.cu_seqlens.astype(np.int32)).cuda()
        outs = []
        for flat in (1, 2):
            st, y, mean, rstd = shaped_forward(base + (clusters, int(case % 2), flat), x, shift, scale, cu, inp.B, inp.T, D)
            assert st == 0, lnmod.lnmod_status_string(st)
            torch.cuda.synchronize()
            outs.append((y, mean, rstd))
        for a, b in zip(*outs):
            assert torch.equal(a, b)
        y64, mean64, rstd64 = oracle.forward(inp.x, inp.shift, inp.scale, inp.workload.eps,
                                             cu=inp.cu_seqlens.astype(np.int64))
        check_io_tensor("y", outs[0][0], y64, "bf16")
        check_stats(outs[0][1], outs[0][2], mean64, rstd64)


def test_uncompiled_shape_fails_and_no_shape_is_the_operator_librarys_launch():
    inp = synth.make_inputs(2, S=1000)
    assert inp.D == 5120
    x, dy = to_device(inp.x, "bf16"), to_device(inp.dy, "bf16")
    shift, scale = to_device(inp.shift, "bf16"), to_device(inp.scale, "bf16")
    y0, mean0, rstd0 = lnmod.forward(x.view(1, 1000, inp.D), shift, scale)
    dx0, dsh0, dsc0 = lnmod.backward(dy.view(1, 1000, inp.D), x.view(1, 1000, inp.D), scale, mean0, rstd0)
    torch.cuda.synchronize()
    st, _, _, _ = shaped_forward((7, 2, 1, 1), x, shift, scale, None, 1, 1000, inp.D)       # no 7-wave kernel
    assert st == lnmod.LNMOD_ELAUNCH
    st, _, _, _ = shaped_forward((2, 2, 1, 4), x, shift, scale, None, 1, 1000, inp.D)       # 256 of 640 chunks
    assert st == lnmod.LNMOD_ELAUNCH
    st, y1, mean1, rstd1 = shaped_forward(None, x, shift, scale, None, 1, 1000, inp.D)
    assert st == 0
    st, dx1, dsh1, dsc1 = shaped_backward(None, dy, x, scale, None, 1, 1000, inp.D, mean1, rstd1)
    assert st == 0
    torch.cuda.synchronize()
    assert torch.equal(y0.view_as(y1), y1) and torch.equal(mean0.view_as(mean1), mean1) and torch.equal(rstd0.view_as(rstd1), rstd1)
    assert torch.equal(dx0.view_as(dx1), dx1) and torch.equal(dsh0, dsh1) and torch.equal(dsc0, dsc1)
    # the table's own entry given explicitly is the same launch again
    st, tab = lnmod_tools.lnmod_table_shape(lnmod_tools.LNMOD_FAMILY_FORWARD, inp.D, 0, 1000)
    assert st == 0
    st, y2, _, _ = shaped_forward(tab, x, shift, scale, None, 1, 1000, inp.D)
    torch.cuda.synchronize()
    assert st == 0 and torch.equal(y1, y2)
