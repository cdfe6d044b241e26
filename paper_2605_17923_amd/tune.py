"""Launch-shape sweep: times every candidate (K, VPL, R, per_cu) of one kernel family at one row
width through the same entry points the library's shape tables serve, and prints the fastest
beside the table's entry.  The tables in csrc/lnmod_launch.hpp and the two gated launchers were
filled in from runs of this procedure on MI355X (one sample of about 774 MB per tensor, the size of
the Wan-14B activation).

    python -m paper_2605_17923_amd.tune --family backward --D 5120
    python -m paper_2605_17923_amd.tune --family gated_forward --D 1536 3072 --dtype bf16 --top 8

Candidates cover the row with at most 60 % padding and keep 3 to 16 waves per compute unit; a
combination the library was not compiled with is reported by the launcher (nothing runs) and
skipped.  Needs a GPU and the built library.
"""
from __future__ import annotations

import argparse

import torch

from . import lnmod

FAMILIES = {"forward": lnmod.LNMOD_TUNE_FORWARD, "backward": lnmod.LNMOD_TUNE_BACKWARD,
            "backward_recompute": lnmod.LNMOD_TUNE_BACKWARD_RECOMPUTE,
            "token_forward": lnmod.LNMOD_TUNE_TOKEN_FORWARD, "token_backward": lnmod.LNMOD_TUNE_TOKEN_BACKWARD,
            "gated_forward": lnmod.LNMOD_TUNE_GATED_FORWARD, "gated_backward": lnmod.LNMOD_TUNE_GATED_BACKWARD,
            "qknorm_forward": lnmod.LNMOD_TUNE_QKNORM_FORWARD, "qknorm_backward": lnmod.LNMOD_TUNE_QKNORM_BACKWARD}


def candidates(nchunks: int):
    out = []
    for K in (1, 2, 3, 4, 5, 6, 8, 10, 12, 16):
        for VPL in (1, 2, 3, 4, 6):
            cover = K * VPL * 64
            if cover < nchunks or cover > 1.6 * nchunks + 64:
                continue
            for R in (1, 2):
                for per_cu in (1, 2, 3, 4, 6, 8):
                    if 3 <= K * per_cu <= 16:
                        out.append((K, VPL, R, per_cu))
    return out


def _ok(status, where):
    if status != 0:
        raise lnmod.LnmodError(status, where)


def _time_us(call, iters, warmup):
    for _ in range(warmup):
        call()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(iters):
        call()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e3 / iters


class Case:
    """Buffers of one (family, D, dtype) and the call that runs it once; `run()` returns the status."""

    def __init__(self, family: str, D: int, dtype: torch.dtype, tensor_bytes: float):
        dev = "cuda"
        self.family, self.D = family, D
        self.code = 0 if dtype == torch.bfloat16 else 1
        T = self.T = max(8192, int(tensor_bytes // (D * dtype.itemsize)))
        big = lambda: torch.randn(T, D, device=dev).to(dtype)       # noqa: E731
        tok = family.startswith("token")
        mrows = T if tok else 1
        self.x, self.out = big(), torch.empty(T, D, device=dev, dtype=dtype)
        self.shift = torch.zeros(mrows, D, device=dev, dtype=dtype)
        self.scale = torch.zeros(mrows, D, device=dev, dtype=dtype)
        self.mean, self.rstd = torch.empty(T, device=dev), torch.empty(T, device=dev)
        if "backward" in family:
            self.dy = big()
            pdt = dtype if tok else torch.float32
            self.dshift = torch.empty(mrows, D, device=dev, dtype=pdt)
            self.dscale = torch.empty(mrows, D, device=dev, dtype=pdt)
        if family.startswith("gated"):
            self.u, self.gate = big(), torch.zeros(1, D, device=dev, dtype=dtype)
            self.out2 = torch.empty(T, D, device=dev, dtype=dtype)
            if "backward" in family:
                self.dh, self.dgate = big(), torch.empty(1, D, device=dev)
        if family.startswith("qknorm"):          # q = x, k = u; rstd of both from the forward below
            self.u, self.out2 = big(), torch.empty(T, D, device=dev, dtype=dtype)
            self.wq, self.wk = (torch.ones(D, device=dev, dtype=dtype) for _ in range(2))
            self.rstd2 = torch.empty(T, device=dev)
            self.dwq, self.dwk = torch.empty(D, device=dev), torch.empty(D, device=dev)
            if "backward" in family:
                self.dh = big()
            _ok(lnmod.lnmod_qknorm_forward(self.x, self.u, self.wq, self.wk, T, D, 1e-6, self._st(), self.out,
                                           self.out2, self.rstd, self.rstd2, self.code), "lnmod_qknorm_forward")
        # statistics for the backward families, from the forward with the table's shape
        st = lnmod.lnmod_forward(self.x, self.shift[:1], self.scale[:1], 1, T, D, 1e-6, self._st(), self.out,
                                 self.mean, self.rstd, self.code, 0)
        _ok(st, "lnmod_forward")
        torch.cuda.synchronize()
        self.ws = None
        self.prepare()

    def prepare(self):
        """The backward workspace follows the launch shape: call after every change of it."""
        if self.family in ("backward", "backward_recompute"):
            self.ws = lnmod.workspace(1, self.T, self.D, "cuda")
        elif self.family == "gated_backward":
            self.ws = lnmod.gated_workspace(1, self.T, self.D, "cuda")
        elif self.family == "qknorm_backward":
            n = lnmod.lnmod_qknorm_backward_workspace_bytes(self.T, self.D)
            self.ws = torch.empty(max(n, 16), dtype=torch.uint8, device="cuda")

    @staticmethod
    def _st():
        return torch.cuda.current_stream().cuda_stream

    def run(self) -> int:
        f, T, D, c, s = self.family, self.T, self.D, self.code, self._st()
        if f == "forward":
            return lnmod.lnmod_forward(self.x, self.shift, self.scale, 1, T, D, 1e-6, s, self.out, self.mean,
                                       self.rstd, c, 0)
        if f == "token_forward":
            return lnmod.lnmod_forward(self.x, self.shift, self.scale, 1, T, D, 1e-6, s, self.out, self.mean,
                                       self.rstd, c, 1)
        if f in ("backward", "backward_recompute"):
            ws = self.ws
            m, r = (self.mean, self.rstd) if f == "backward" else (None, None)
            return lnmod.lnmod_backward(self.dy, self.x, None, self.scale, 1, T, D, 1e-6, s, m, r, self.out,
                                        self.dshift, self.dscale, ws, ws.numel(), c, 0)
        if f == "token_backward":
            return lnmod.lnmod_backward(self.dy, self.x, None, self.scale, 1, T, D, 1e-6, s, self.mean, self.rstd,
                                        self.out, self.dshift, self.dscale, None, 0, c, 1)
        if f == "gated_forward":
            return lnmod.lnmod_gated_forward(self.x, self.u, self.gate, self.shift, self.scale, None, 1, T, D, 1e-6,
                                             s, self.out, self.out2, self.mean, self.rstd, c)
        if f == "qknorm_forward":
            return lnmod.lnmod_qknorm_forward(self.x, self.u, self.wq, self.wk, T, D, 1e-6, s, self.out, self.out2,
                                              self.rstd, self.rstd2, c)
        ws = self.ws
        if f == "qknorm_backward":
            return lnmod.lnmod_qknorm_backward(self.dy, self.dh, self.x, self.u, self.wq, self.wk, T, D, 1e-6, s,
                                               self.rstd, self.rstd2, self.out, self.out2, self.dwq, self.dwk, ws,
                                               ws.numel(), c)
        return lnmod.lnmod_gated_backward(self.dy, self.dh, self.x, self.u, self.gate, self.scale, None, 1, T, D,
                                          1e-6, s, self.mean, self.rstd, self.out, self.out2, self.dgate,
                                          self.dshift, self.dscale, ws, ws.numel(), c)


def sweep(family: str, D: int, dtype: torch.dtype, tensor_bytes: float, iters: int, warmup: int):
    """Returns (table shape, its time in us before and after the sweep, [(shape, us)] sorted by time)."""
    fam = FAMILIES[family]
    case = Case(family, D, dtype, tensor_bytes)
    st, table = lnmod.lnmod_tuning_table_shape(fam, D, case.code)
    _ok(st, "lnmod_tuning_table_shape")
    results = []
    try:
        _ok(case.run(), family)
        for _ in range(100):                       # bring the clocks up before the first number
            case.run()
        before = _time_us(case.run, iters, warmup)
        for shape in candidates(D // (8 if case.code == 0 else 4)):
            if lnmod.lnmod_tuning_set_shape(fam, *shape) != 0:
                continue
            case.prepare()
            if case.run() != 0:                    # not compiled for this family and type: nothing ran
                continue
            results.append((shape, _time_us(case.run, iters, warmup)))
    finally:
        lnmod.lnmod_tuning_set_shape(fam, 0, 0, 0, 0)
    case.prepare()
    after = _time_us(case.run, iters, warmup)
    torch.cuda.synchronize()
    return table, before, after, sorted(results, key=lambda r: r[1])


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--family", required=True, choices=sorted(FAMILIES))
    ap.add_argument("--D", type=int, nargs="+", required=True)
    ap.add_argument("--dtype", choices=("bf16", "fp32"), default="bf16")
    ap.add_argument("--bytes", type=float, default=774e6, help="size of one [T, D] tensor (default: 774 MB)")
    ap.add_argument("--iters", type=int, default=12)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--top", type=int, default=5)
    args = ap.parse_args(argv)
    if not torch.cuda.is_available():
        raise SystemExit("the shape sweep needs a GPU")
    dtype = torch.bfloat16 if args.dtype == "bf16" else torch.float32
    for D in args.D:
        table, before, after, res = sweep(args.family, D, dtype, args.bytes, args.iters, args.warmup)
        print("%s D=%d %s: table %s %.1f us (after the sweep %.1f us); %d candidates ran"
              % (args.family, D, args.dtype, table, before, after, len(res)), flush=True)
        for shape, us in res[:args.top]:
            print("    %-16s %.1f us" % (shape, us), flush=True)
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
