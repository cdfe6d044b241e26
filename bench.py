#!/usr/bin/env python3
"""Benchmark of the fused LayerNorm-Modulate hot path on one MI355X.

A step is one pass of the whole hot path over one batch of the Wan-14B-shaped workload
(bf16, B=1, S=75600 tokens, D=5120): lnmod_forward (y, mean, rstd) followed by lnmod_backward
(dx, dshift, dscale; the fused dx+partials kernel and its fixed-order second pass).  Inputs are
synthetic, generated on the device from a seeded generator with the workload's distributions,
and resident in HBM before the timed region.

Prints ONE JSON line.  `value` is algorithmic HBM bytes of a step / wall time of a step
(GB/s); `roofline` describes the dominant launch (the backward) and `roofline_fwd` the forward
kernel, both from HIP events recorded on the launch stream inside the timed region;
`cpu_baseline` is the float64 CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X published HBM3E bandwidth

# HBM traffic per launch measured with rocprofv3 --pmc (FETCH_SIZE, then WRITE_SIZE), each scaled
# by the same counter's reading for lnmod_copy of known size.  The figures live in a tracked table
# beside the summaries they come from; every row names the launch it was measured on (kernel
# instantiation, grid, slots: the text lnmod_describe_launch gives), and a row whose launch is not
# the one the library makes today is not used: `traffic` is then null instead of stale.
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_table.txt")


def measured_traffic(entry, launch):
    """HBM bytes per launch for `entry` ('forward' / 'backward' of the headline workload) from the
    tracked table, or None when the table has no row for exactly this launch."""
    try:
        rows = open(TRAFFIC_TABLE).read().splitlines()
    except OSError:
        return None
    for line in rows:
        if line.startswith("#") or "|" not in line:
            continue
        cols = [c.strip() for c in line.split("|")]
        if len(cols) >= 3 and cols[0] == entry and cols[1] == launch:
            return int(cols[2])
    return None


def algorithmic_bytes(T, D, elem):
    """Bytes the method itself must move per launch.  Forward: x in, y out, mean+rstd out.
    Backward: dy, x in, dx out, mean+rstd in (the per-block partial sums and the [B,2,D] result
    are excluded: they are this implementation's choice, about 1 % extra)."""
    fwd = T * (2 * D * elem + 8)
    bwd = T * (3 * D * elem + 8)
    return fwd, bwd


def make_device_inputs(T, D, seed, device):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    x = torch.randn(T, D, generator=g, device=device) * 2.0 + 0.5
    mask = torch.rand(T, D, generator=g, device=device) < 1e-3
    x = torch.where(mask, x * 50.0, x).to(torch.bfloat16)
    del mask
    dy = torch.randn(T, D, generator=g, device=device).to(torch.bfloat16)
    shift = (0.1 * torch.randn(1, D, generator=g, device=device)).to(torch.bfloat16)
    scale = (0.1 * torch.randn(1, D, generator=g, device=device)).to(torch.bfloat16)
    return x, dy, shift, scale


def cpu_baseline(D, sample_tokens, repeats=3):
    """The oracle as it stands, forward + backward on `sample_tokens` tokens of the workload
    (host-generated from the workload's recipe), median of `repeats` runs."""
    import oracle
    from paper_2605_17923_amd import synth
    inp = synth.make_inputs(2, S=sample_tokens)
    oracle.forward(inp.x[:64], inp.shift, inp.scale, 1e-6, B=1, S=64)      # load + warm the library
    times = []
    for _ in range(repeats):
        t0 = time.perf_counter()
        oracle.forward(inp.x, inp.shift, inp.scale, 1e-6, B=1, S=sample_tokens)
        oracle.backward(inp.dy, inp.x, inp.scale, 1e-6, B=1, S=sample_tokens)
        times.append(time.perf_counter() - t0)
    dt = sorted(times)[len(times) // 2]
    fwd_b, bwd_b = algorithmic_bytes(sample_tokens, D, 2)
    cores = oracle.num_threads()
    one = None
    if cores > 1:                                   # the same work on one thread, once
        oracle.set_num_threads(1)
        try:
            t0 = time.perf_counter()
            oracle.forward(inp.x, inp.shift, inp.scale, 1e-6, B=1, S=sample_tokens)
            oracle.backward(inp.dy, inp.x, inp.scale, 1e-6, B=1, S=sample_tokens)
            t1 = time.perf_counter() - t0
        finally:
            oracle.set_num_threads(cores)
        one = {"value": round((fwd_b + bwd_b) / t1 / 1e9, 3), "unit": "GB/s", "cores": 1,
               "tokens_per_s": round(sample_tokens / t1), "seconds": round(t1, 3)}
    # the forward-only workload [1] (bf16 B=1 S=32760 D=1536), all cores, median of 3
    inp1 = synth.make_inputs(1)
    t1s = []
    for _ in range(repeats):
        t0 = time.perf_counter()
        oracle.forward(inp1.x, inp1.shift, inp1.scale, 1e-6, B=1, S=inp1.T)
        t1s.append(time.perf_counter() - t0)
    d1 = sorted(t1s)[len(t1s) // 2]
    cfg1 = {"workload": "configs[1] forward, 32760 x 1536", "value": round(inp1.T * (4 * inp1.D + 8) / d1 / 1e9, 3),
            "unit": "GB/s", "cores": cores, "tokens_per_s": round(inp1.T / d1), "seconds": round(d1, 4)}
    return {"value": round((fwd_b + bwd_b) / dt / 1e9, 3), "unit": "GB/s", "cores": cores,
            "kind": "oracle", "tokens_per_s": round(sample_tokens / dt), "seconds": round(dt, 3),
            "config1_forward": cfg1,
            "sample": "%d of the workload's 75600 tokens (fwd+bwd, float64 C, OpenMP over rows), "
                      "median of %d runs" % (sample_tokens, repeats),
            "one_thread": one}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--cpu-sample-tokens", type=int, default=75600)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run lnmod_copy on a buffer of the workload's size (a kernel of known "
                         "traffic for scaling the rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--gated-only", action="store_true",
                    help="only time the gated residual + LayerNorm-Modulate and the Q-Norm + K-Norm "
                         "fusions on the workload's shape (for profiling their kernels; not the "
                         "headline metric)")
    ap.add_argument("--only-workload", type=int, choices=(1, 3, 4), default=None,
                    help="only run forward and backward of workload configs[N] (--steps launches each), for "
                         "profiling its kernels under rocprofv3; not the headline metric")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the copy ceiling, the unfused comparison and the D=1536 forward")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the operator has no cross-GPU step); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_17923_amd import lnmod, lnmod_tools

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    lnmod.library()
    lnmod_tools.library()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    B, S, D = 1, 75600, 5120
    T = B * S
    if args.calibrate_copy:
        src = torch.zeros(T, D, dtype=torch.bfloat16, device=dev)
        dst = torch.empty_like(src)
        stream = torch.cuda.current_stream()
        nbytes = src.numel() * 2
        ms = _time_ms(torch, stream, lambda: lnmod_tools.lnmod_copy(src, dst, nbytes, stream.cuda_stream), iters=args.steps)
        print(json.dumps({"kernel": "copy16_kernel", "bytes_read": nbytes, "bytes_written": nbytes,
                          "avg_launch_us": round(ms * 1e3, 2), "GBs": _gbs(2 * nbytes, ms)}))
        return
    if args.gated_only:
        stream = torch.cuda.current_stream()
        print(json.dumps({"gated": _run_gated(lnmod, lnmod_tools, torch, stream, stream.cuda_stream, dev, T, D,
                                              iters=args.steps),
                          "qknorm": _run_qknorm(lnmod, torch, stream, stream.cuda_stream, dev, T, D,
                                                iters=args.steps),
                          "qknorm_per_head": _run_qknorm(lnmod, torch, stream, stream.cuda_stream, dev,
                                                         T * (D // 128), 128, iters=args.steps)}))
        return
    if args.only_workload is not None:
        stream = torch.cuda.current_stream()
        print(json.dumps(other_workload(args.only_workload, lnmod, torch, stream, stream.cuda_stream, dev,
                                        iters=args.steps)))
        return
    x, dy, shift, scale = make_device_inputs(T, D, 1003, dev)
    y, dx = torch.empty_like(x), torch.empty_like(x)
    mean = torch.empty(T, dtype=torch.float32, device=dev)
    rstd = torch.empty(T, dtype=torch.float32, device=dev)
    dshift = torch.empty(B, D, dtype=torch.float32, device=dev)
    dscale = torch.empty(B, D, dtype=torch.float32, device=dev)
    ws = lnmod.workspace(B, T, D, dev)
    stream = torch.cuda.current_stream()
    st = stream.cuda_stream
    BF16, PER_SAMPLE = lnmod.LNMOD_BF16, lnmod.LNMOD_PER_SAMPLE

    def fwd():
        rc = lnmod.lnmod_forward(x, shift, scale, B, S, D, 1e-6, st, y, mean, rstd, BF16, PER_SAMPLE)
        assert rc == 0, lnmod.lnmod_status_string(rc)

    def bwd():
        rc = lnmod.lnmod_backward(dy, x, None, scale, B, S, D, 1e-6, st, mean, rstd, dx, dshift,
                                  dscale, ws, ws.numel(), BF16, PER_SAMPLE)
        assert rc == 0, lnmod.lnmod_status_string(rc)

    conditioning = condition(torch, stream, lambda: (fwd(), bwd()))

    for _ in range(args.warmup):
        fwd()
        bwd()
    torch.cuda.synchronize()

    K = args.steps
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(K)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K):
        ev[k][0].record(stream)
        fwd()
        ev[k][1].record(stream)
        bwd()
        ev[k][2].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    fwd_all = sorted(e[0].elapsed_time(e[1]) for e in ev)
    bwd_all = sorted(e[1].elapsed_time(e[2]) for e in ev)
    step_all = sorted(e[0].elapsed_time(e[2]) for e in ev)
    fwd_ms = sum(fwd_all) / K
    bwd_ms = sum(bwd_all) / K
    ms_per_step = wall * 1e3 / K
    fwd_b, bwd_b = algorithmic_bytes(T, D, 2)
    value = (fwd_b + bwd_b) / (ms_per_step * 1e-3) / 1e9
    median_step_ms = step_all[K // 2]
    fwd_launch = lnmod_tools.lnmod_describe_launch(False, None, B, S, False, D, BF16, PER_SAMPLE)
    bwd_launch = lnmod_tools.lnmod_describe_launch(True, None, B, S, False, D, BF16, PER_SAMPLE)

    def roof(nbytes, ms, kernel, launch, traffic, all_ms):
        a = nbytes / (ms * 1e-3) / 1e9
        return {"bound": "hbm", "kernel": kernel, "launch": launch, "achieved": round(a, 1), "peak": PEAK_HBM_GBS,
                "unit": "GB/s", "frac": round(a / PEAK_HBM_GBS, 4), "traffic": traffic,
                "avg_launch_us": round(ms * 1e3, 2), "median_launch_us": round(all_ms[len(all_ms) // 2] * 1e3, 2),
                "min_launch_us": round(all_ms[0] * 1e3, 2), "algorithmic_bytes": nbytes,
                "tokens_per_s": round(T / (ms * 1e-3))}

    out = {
        "metric": "achieved HBM GB/s (% of MI355X peak) + tokens/s, LN-Modulate fwd/bwd",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "configs[2] Wan-14B-shaped fwd+bwd: bf16 I/O, B=1, S=75600, D=5120, "
                               "x~N(0.5,2) with 0.1% x50 outliers, per-sample shift/scale, eps=1e-6",
                   "io_dtype": "bf16", "B": B, "S": S, "D": D},
        "frac_of_peak": round(value / PEAK_HBM_GBS, 4),
        "tokens_per_s": round(T / (ms_per_step * 1e-3)),
        "median_ms_per_step": round(median_step_ms, 4),
        "value_at_median_step": round((fwd_b + bwd_b) / (median_step_ms * 1e-3) / 1e9, 1),
        "conditioning": conditioning,
        "roofline": roof(bwd_b, bwd_ms, "lnmod_backward = bwd_seg_kernel + bwd_reduce_kernel "
                                        "(durations summed)", bwd_launch,
                         measured_traffic("backward", bwd_launch), bwd_all),
        "roofline_fwd": roof(fwd_b, fwd_ms, "fwd_split_kernel", fwd_launch,
                             measured_traffic("forward", fwd_launch), fwd_all),
    }

    if not args.no_extras:
        out["extras"] = extras(lnmod, lnmod_tools, torch, x, dy, y, shift, scale, mean, rstd, T, D, st, stream)
        # backward that forms the statistics again from x (no mean/rstd kept between the passes),
        # next to the saved-statistics backward timed the same way (back-to-back launches)
        def bwd_rc():
            rc = lnmod.lnmod_backward(dy, x, None, scale, B, S, D, 1e-6, st, None, None, dx, dshift,
                                      dscale, ws, ws.numel(), BF16, PER_SAMPLE)
            assert rc == 0, lnmod.lnmod_status_string(rc)
        sv_ms = _time_ms(torch, stream, bwd, iters=40, warm=5)
        rc_ms = _time_ms(torch, stream, bwd_rc, iters=40, warm=5)
        sv2_ms = _time_ms(torch, stream, bwd, iters=40, warm=5)
        # the same step replayed from a HIP graph of 20 (no host work and no gaps between launches)
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            cs = torch.cuda.current_stream().cuda_stream
            for _ in range(20):
                rc = lnmod.lnmod_forward(x, shift, scale, B, S, D, 1e-6, cs, y, mean, rstd, BF16, PER_SAMPLE)
                rc |= lnmod.lnmod_backward(dy, x, None, scale, B, S, D, 1e-6, cs, mean, rstd, dx, dshift, dscale, ws,
                                           ws.numel(), BF16, PER_SAMPLE)
                assert rc == 0, lnmod.lnmod_status_string(rc)
        torch.cuda.synchronize()
        g_ms = _time_ms(torch, torch.cuda.current_stream(), gr.replay, iters=5, warm=2) / 20
        out["extras"]["step_in_hip_graph"] = {"ms_per_step": round(g_ms, 4), "GBs": _gbs(fwd_b + bwd_b, g_ms)}
        del gr
        out["extras"]["bwd_recompute_stats"] = {
            "recompute_us": round(rc_ms * 1e3, 1), "recompute_GBs": _gbs(T * 6 * D, rc_ms),
            "saved_stats_back_to_back_us": [round(sv_ms * 1e3, 1), round(sv2_ms * 1e3, 1)]}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(D, args.cpu_sample_tokens)
    print(json.dumps(out))


def condition(torch, stream, step, group=8, tol=0.01, min_ms=100.0, cap_ms=300.0):
    """Untimed, bounded conditioning before the warm-up and the timed steps.  A process that has
    just started finds the GPU at idle clocks: the first steps run up to 40 % slow, speed up over
    some tens of milliseconds, sit on a plateau about 5 % above the final rate for another ten and
    only then reach it (per-step kernel times of such a run are in profiles/), which `warmup`
    steps of 0.6 ms do not cover.  The step is run in groups of `group` for at least `min_ms` of
    GPU time; after that the phase ends as soon as a group's mean step time is no longer more than
    `tol` below the previous group's, or after `cap_ms`.  Nothing measured here enters the
    reported figures; what was done is reported beside them."""
    means = []
    spent = 0.0
    reason = "cap"
    while spent < cap_ms:
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(group):
            step()
        b.record(stream)
        torch.cuda.synchronize()
        ms = a.elapsed_time(b)
        spent += ms
        means.append(ms / group)
        if spent >= min_ms and len(means) >= 2 and means[-1] >= means[-2] * (1.0 - tol):
            reason = "settled"
            break
    return {"steps": group * len(means), "gpu_ms": round(spent, 2), "ended": reason,
            "first_group_ms_per_step": round(means[0], 4), "last_group_ms_per_step": round(means[-1], 4)}


def _time_ms(torch, stream, fn, iters=20, warm=3, settle_ms=30.0):
    """Mean time of `iters` calls of fn (events on the launch stream).  Before the warm-up the call is
    repeated, untimed, until its rate has settled (see condition(); at least `settle_ms` of GPU time):
    between two measurements of this file the host builds tensors, and a GPU left idle for some tens
    of milliseconds drops its clocks (50 ms pauses cost the forward 26 %, and the 20 launches of a
    measurement taken right after tensor setup ran 580 ... 530 us where the settled rate is 512)."""
    if settle_ms > 0:
        condition(torch, stream, fn, min_ms=settle_ms, cap_ms=250.0)
    for _ in range(warm):
        fn()
    a = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
    a[0].record(stream)
    for i in range(iters):
        fn()
        a[i + 1].record(stream)
    torch.cuda.synchronize()
    return sum(a[i].elapsed_time(a[i + 1]) for i in range(iters)) / iters


def _gbs(nbytes, ms):
    return round(nbytes / (ms * 1e-3) / 1e9, 1)


def _randn_bf16(torch, g, shape, dev, std=1.0, mean=0.0):
    return (torch.randn(*shape, generator=g, device=dev) * std + mean).to(torch.bfloat16)


def other_workload(index, lnmod, torch, stream, st, dev, iters=20):
    """Workloads configs[1], [3], [4] in the shapes the workload list gives them."""
    PS, PT = lnmod.LNMOD_PER_SAMPLE, lnmod.LNMOD_PER_TOKEN
    if index == 1:
        # 201 MB per forward is less than the 256 MB of memory-side cache: three buffer sets are rotated so that
        # a set has been pushed out (by 400 MB of other traffic) before it is used again.  The same launches on
        # one set, for comparison: equal times mean the cache was not helping in the first place.
        res = _run_workload(lnmod, torch, stream, st, dev, "configs[1] Wan-1.3B B=1 S=32760 D=1536 (3 buffer sets "
                            "rotated)", 1, 32760, 1536, PS, rotate=3, seed=1002, graph=True, iters=iters)
        one = _run_workload(lnmod, torch, stream, st, dev, "", 1, 32760, 1536, PS, rotate=1, seed=1002, iters=iters)
        res["fwd_us_one_buffer_set"], res["bwd_us_one_buffer_set"] = one["fwd_us"], one["bwd_us"]
        return res
    if index == 3:
        return _run_workload(lnmod, torch, stream, st, dev, "configs[3] per-token B=2 S=32760 D=5120", 2, 32760, 5120,
                             PT, seed=1004, iters=iters)
    from paper_2605_17923_amd import synth
    lengths, _ = synth.varlen_lengths()
    return _run_workload(lnmod, torch, stream, st, dev, "configs[4] varlen 24 segments T=%d D=5120" % sum(lengths),
                         24, 0, 5120, PS, lengths=lengths, seed=1005, iters=iters)


def _run_workload(lnmod, torch, stream, st, dev, name, B, S, D, mod, lengths=None, rotate=1, seed=1, fp32=False,
                  graph=False, iters=20):
    """Forward and backward of one workload shape (bf16, or fp32 I/O), timed with events on the launch stream.
    `rotate` > 1 cycles through that many independent buffer sets so that a workload smaller
    than the 256 MB Infinity Cache still streams from HBM."""
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    io_dt = torch.float32 if fp32 else torch.bfloat16
    code = lnmod.LNMOD_F32 if fp32 else lnmod.LNMOD_BF16
    elem = 4 if fp32 else 2
    T = int(sum(lengths)) if lengths is not None else B * S
    nseg = len(lengths) if lengths is not None else B
    per_token = mod == lnmod.LNMOD_PER_TOKEN
    mrows = T if per_token else nseg
    sets = []
    for _ in range(rotate):
        x = _randn_bf16(torch, g, (T, D), dev).to(io_dt)
        dy = _randn_bf16(torch, g, (T, D), dev).to(io_dt)
        sh = _randn_bf16(torch, g, (mrows, D), dev, 0.1).to(io_dt)
        sc = _randn_bf16(torch, g, (mrows, D), dev, 0.1).to(io_dt)
        y, dx = torch.empty_like(x), torch.empty_like(x)
        if per_token:
            dsh, dsc = torch.empty_like(x), torch.empty_like(x)
        else:
            dsh = torch.empty(nseg, D, dtype=torch.float32, device=dev)
            dsc = torch.empty(nseg, D, dtype=torch.float32, device=dev)
        sets.append((x, dy, sh, sc, y, dx, dsh, dsc))
    mean = torch.empty(T, dtype=torch.float32, device=dev)
    rstd = torch.empty(T, dtype=torch.float32, device=dev)
    ws = lnmod.workspace(nseg, T, D, dev)
    cu = None
    if lengths is not None:
        import itertools
        cu = torch.tensor([0] + list(itertools.accumulate(lengths)), dtype=torch.int32, device=dev)
    state = {"i": 0}

    def pick():
        state["i"] = (state["i"] + 1) % rotate
        return sets[state["i"]]

    def fwd(s=st):
        x, dy, sh, sc, y, dx, dsh, dsc = pick()
        if cu is not None:
            rc = lnmod.lnmod_forward_varlen(x, sh, sc, cu, nseg, T, D, 1e-6, s, y, mean, rstd, code)
        else:
            rc = lnmod.lnmod_forward(x, sh, sc, B, S, D, 1e-6, s, y, mean, rstd, code, mod)
        assert rc == 0, lnmod.lnmod_status_string(rc)

    def bwd(s=st):
        x, dy, sh, sc, y, dx, dsh, dsc = pick()
        if cu is not None:
            rc = lnmod.lnmod_backward_varlen(dy, x, None, sc, cu, nseg, T, D, 1e-6, s, mean, rstd, dx, dsh,
                                             dsc, ws, ws.numel(), code)
        else:
            rc = lnmod.lnmod_backward(dy, x, None, sc, B, S, D, 1e-6, s, mean, rstd, dx, dsh, dsc, ws,
                                      ws.numel(), code, mod)
        assert rc == 0, lnmod.lnmod_status_string(rc)

    fwd()
    torch.cuda.synchronize()
    f_ms = _time_ms(torch, stream, fwd, iters=iters)
    b_ms = _time_ms(torch, stream, bwd, iters=iters)
    mod_bytes = 2 * D * elem                    # shift + scale, or scale + two per-token outputs
    fwd_b = T * (2 * elem * D + 8) + (T * mod_bytes if per_token else 0)
    bwd_b = T * (3 * elem * D + 8) + (T * 3 * D * elem if per_token else 0)
    out = {"workload": name, "tokens": T, "D": D,
           "fwd_us": round(f_ms * 1e3, 1), "fwd_GBs": _gbs(fwd_b, f_ms), "fwd_frac": round(_gbs(fwd_b, f_ms) / PEAK_HBM_GBS, 3),
           "bwd_us": round(b_ms * 1e3, 1), "bwd_GBs": _gbs(bwd_b, b_ms), "bwd_frac": round(_gbs(bwd_b, b_ms) / PEAK_HBM_GBS, 3)}
    if graph:
        # a problem this short pays for the gaps between launches: the same launches replayed
        # from a HIP graph of 40 (the library allocates nothing and records no memset, so its calls
        # can be captured as they are)
        for key, fn in (("fwd_us_in_hip_graph", fwd), ("bwd_us_in_hip_graph", bwd)):
            n = 40
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr):
                for _ in range(n):
                    fn(torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            ms = _time_ms(torch, torch.cuda.current_stream(), gr.replay, iters=10, warm=3)
            out[key] = round(ms * 1e3 / n, 1)
            del gr
    return out


def _run_gated(lnmod, lnmod_tools, torch, stream, st, dev, T, D, iters=20):
    """The gated residual + LayerNorm-Modulate fusion on the workload's shape (bf16, one sample):
    fused forward against the unfused chain (residual kernel, then lnmod_forward on h), and the
    fused backward.  Algorithmic bytes per token: forward 8D+8 (x, u in; h, y, statistics out),
    backward 12D+8 (dy, dh, h, u, statistics in; dx, du out)."""
    g = torch.Generator(device=dev)
    g.manual_seed(77)
    x, u, dy, dh = (_randn_bf16(torch, g, (T, D), dev) for _ in range(4))
    gate, shift, scale = (_randn_bf16(torch, g, (1, D), dev, 0.2) for _ in range(3))
    h, y, dx, du = (torch.empty_like(x) for _ in range(4))
    mean = torch.empty(T, dtype=torch.float32, device=dev)
    rstd = torch.empty(T, dtype=torch.float32, device=dev)
    dg, dsh, dsc = (torch.empty(1, D, dtype=torch.float32, device=dev) for _ in range(3))
    ws = lnmod.gated_workspace(1, T, D, dev)
    BF = lnmod.LNMOD_BF16

    def fused_fwd():
        rc = lnmod.lnmod_gated_forward(x, u, gate, shift, scale, None, 1, T, D, 1e-6, st, h, y, mean, rstd, BF)
        assert rc == 0, lnmod.lnmod_status_string(rc)

    def unfused_fwd():
        rc = lnmod_tools.lnmod_gate_residual(x, u, gate, 1, T, D, st, h, BF)
        assert rc == 0, lnmod.lnmod_status_string(rc)
        rc = lnmod.lnmod_forward(h, shift, scale, 1, T, D, 1e-6, st, y, mean, rstd, BF, lnmod.LNMOD_PER_SAMPLE)
        assert rc == 0, lnmod.lnmod_status_string(rc)

    def fused_bwd():
        rc = lnmod.lnmod_gated_backward(dy, dh, h, u, gate, scale, None, 1, T, D, 1e-6, st, mean, rstd, dx, du,
                                        dg, dsh, dsc, ws, ws.numel(), BF)
        assert rc == 0, lnmod.lnmod_status_string(rc)

    f_ms = _time_ms(torch, stream, fused_fwd, iters=iters)
    uf_ms = _time_ms(torch, stream, unfused_fwd, iters=iters)
    b_ms = _time_ms(torch, stream, fused_bwd, iters=iters)
    fwd_b, bwd_b = T * (8 * D + 8), T * (12 * D + 8)
    return {"workload": "gated residual + LN-Modulate, bf16 B=1 S=%d D=%d" % (T, D),
            "fwd_us": round(f_ms * 1e3, 1), "fwd_GBs": _gbs(fwd_b, f_ms), "fwd_frac": round(_gbs(fwd_b, f_ms) / PEAK_HBM_GBS, 3),
            "unfused_fwd_us": round(uf_ms * 1e3, 1), "fused_vs_unfused_fwd_speedup": round(uf_ms / f_ms, 3),
            "bwd_us": round(b_ms * 1e3, 1), "bwd_GBs": _gbs(bwd_b, b_ms), "bwd_frac": round(_gbs(bwd_b, b_ms) / PEAK_HBM_GBS, 3)}


def _run_qknorm(lnmod, torch, stream, st, dev, T, D, iters=20):
    """The fused Q-Norm + K-Norm on the workload's shape (bf16): both tensors in one launch.
    Algorithmic bytes per token: forward 8D+8 (q, k in; both out; two rstd), backward 12D+8."""
    g = torch.Generator(device=dev)
    g.manual_seed(78)
    q, k, dqo, dko = (_randn_bf16(torch, g, (T, D), dev) for _ in range(4))
    wq, wk = (_randn_bf16(torch, g, (D,), dev, 0.1, 1.0) for _ in range(2))
    q_out, k_out, dq, dk = (torch.empty_like(q) for _ in range(4))
    rq = torch.empty(T, dtype=torch.float32, device=dev)
    rk = torch.empty(T, dtype=torch.float32, device=dev)
    dwq, dwk = (torch.empty(D, dtype=torch.float32, device=dev) for _ in range(2))
    ws = torch.empty(max(lnmod.lnmod_qknorm_backward_workspace_bytes(T, D), 16), dtype=torch.uint8, device=dev)
    BF = lnmod.LNMOD_BF16

    def fwd():
        rc = lnmod.lnmod_qknorm_forward(q, k, wq, wk, T, D, 1e-6, st, q_out, k_out, rq, rk, BF)
        assert rc == 0, lnmod.lnmod_status_string(rc)

    def bwd():
        rc = lnmod.lnmod_qknorm_backward(dqo, dko, q, k, wq, wk, T, D, 1e-6, st, rq, rk, dq, dk, dwq, dwk,
                                         ws, ws.numel(), BF)
        assert rc == 0, lnmod.lnmod_status_string(rc)

    f_ms = _time_ms(torch, stream, fwd, iters=iters)
    b_ms = _time_ms(torch, stream, bwd, iters=iters)
    fwd_b, bwd_b = T * (8 * D + 8), T * (12 * D + 8)
    return {"workload": "Q-Norm + K-Norm, bf16 N=%d D=%d" % (T, D),
            "fwd_us": round(f_ms * 1e3, 1), "fwd_GBs": _gbs(fwd_b, f_ms), "fwd_frac": round(_gbs(fwd_b, f_ms) / PEAK_HBM_GBS, 3),
            "bwd_us": round(b_ms * 1e3, 1), "bwd_GBs": _gbs(bwd_b, b_ms), "bwd_frac": round(_gbs(bwd_b, b_ms) / PEAK_HBM_GBS, 3)}


def probe_ceilings(lnmod_tools, torch, stream, st, bufs, nbytes):
    """What the memory system gives to the read/write mixtures of the kernels, in the copy's access
    pattern: GB/s of lnmod_stream_probe for (reads, writes) streams of `nbytes` each.  The mixtures:
    reads alone, writes alone, 1R1W (forward), 2R1W (backward), 2R2W (gated forward, Q/K-norm forward),
    3R1W (per-token forward), 3R3W (per-token backward), 4R2W (gated backward, Q/K-norm backward)."""
    res = {}
    for nr, nw in lnmod_tools.PROBE_MIXTURES:
        ins = bufs[:nr]
        outs = bufs[nr:nr + max(nw, 1)]

        def call():
            rc = lnmod_tools.lnmod_stream_probe(ins, outs, nbytes, st, writes=nw)
            assert rc == 0, rc
        ms = _time_ms(torch, stream, call)
        res["%dR%dW" % (nr, nw)] = _gbs((nr + nw) * nbytes, ms)
    return res


def extras(lnmod, lnmod_tools, torch, x, dy, y, shift, scale, mean, rstd, T, D, st, stream):
    """Context figures: a plain copy and the stream probes as the practical bandwidth ceilings, the
    unfused two-kernel forward (LayerNorm -> xhat in HBM -> modulate), the other workload shapes and
    the token counts of the paper's kernel table (Table 2: N = 8k ... 64k) at D = 5120."""
    res = {}
    dev = x.device
    nbytes = x.numel() * 2
    tmp = torch.empty_like(x)
    # the copy's rate moves by up to 20 % with where the two buffers happen to lie: best of three pairings
    pairs = [_gbs(2 * nbytes, _time_ms(torch, stream, lambda s=s_, d=d_: lnmod_tools.lnmod_copy(s, d, nbytes, st)))
             for s_, d_ in ((x, y), (dy, tmp), (x, tmp))]
    res["copy_ceiling_GBs"] = max(pairs)
    res["copy_GBs_by_buffer_pair"] = pairs
    bufs = [x, dy, y, tmp] + [torch.empty_like(x) for _ in range(2)]
    res["stream_ceilings_GBs"] = probe_ceilings(lnmod_tools, torch, stream, st, bufs, nbytes)
    del bufs
    ms_u = _time_ms(torch, stream, lambda: lnmod_tools.lnmod_unfused_forward(
        x, shift, scale, 1, T, D, 1e-6, st, tmp, y, mean, rstd, lnmod.LNMOD_BF16))
    ms_f = _time_ms(torch, stream, lambda: lnmod.lnmod_forward(
        x, shift, scale, 1, T, D, 1e-6, st, y, mean, rstd, lnmod.LNMOD_BF16, lnmod.LNMOD_PER_SAMPLE))
    res["unfused_fwd_us"] = round(ms_u * 1e3, 1)
    res["fused_fwd_us"] = round(ms_f * 1e3, 1)
    res["fused_vs_unfused_fwd_speedup"] = round(ms_u / ms_f, 3)
    del tmp
    PS = lnmod.LNMOD_PER_SAMPLE
    res["workloads"] = [
        other_workload(1, lnmod, torch, stream, st, dev),
        other_workload(3, lnmod, torch, stream, st, dev),
        other_workload(4, lnmod, torch, stream, st, dev),
        _run_workload(lnmod, torch, stream, st, dev, "fp32 I/O B=1 S=37800 D=5120 (the bytes of configs[2])",
                      1, 37800, 5120, PS, seed=1006, fp32=True),
    ]
    res["gated"] = _run_gated(lnmod, lnmod_tools, torch, stream, st, dev, T, D)
    res["qknorm"] = _run_qknorm(lnmod, torch, stream, st, dev, T, D)
    res["qknorm_per_head"] = _run_qknorm(lnmod, torch, stream, st, dev, T * (D // 128), 128)
    # the token counts of the paper's kernel table (Table 2: N = 8k ... 64k), fused kernels at D = 5120 bf16
    grid = []
    for n in range(8000, 64001, 8000):
        r = _run_workload(lnmod, torch, stream, st, dev, "N=%d" % n, 1, n, 5120, PS, seed=n)
        grid.append({"N": n, "fwd_us": r["fwd_us"], "bwd_us": r["bwd_us"]})
    res["paper_table2_grid_D5120"] = grid
    return res


if __name__ == "__main__":
    main()
