"""Seeded synthetic inputs for the LayerNorm-Modulate workloads.

This module only draws random numbers and shapes them; it contains none of the operator's
arithmetic and is the one piece of code that both the GPU tests/benchmark and the CPU oracle's
tests feed from.  Every array is float32 on the host.  For a bf16 workload the values have
already been rounded to bf16 (round to nearest even), so the float32 array is an exact carrier
of what the device sees and of what a float64 reference should read.

The five workloads stand in for the activations of Wan 2.1 DiT blocks (the paper trains on
WebDataset and Koala-36M clips, Sec. 4.1; neither data nor weights are needed because the
operator's cost depends on shapes only):

  0  tiny fp32        B=2, S=256,   D=1536, per-sample modulation, fwd+bwd
  1  Wan-1.3B, bf16   B=1, S=32760, D=1536, per-sample modulation, fwd
  2  Wan-14B,  bf16   B=1, S=75600, D=5120, x ~ N(0.5, std 2) with 0.1 % of entries x50, fwd+bwd
  3  per-token, bf16  B=2, S=32760, D=5120, shift/scale [B,S,D], fwd+bwd
  4  varlen,   bf16   24 packed segments, D=5120, lengths from {1560, 8190, 16380, 32760}
                      with weights .5/.2/.2/.1 and a total of about 150k tokens, fwd+bwd

N(a, b) is read as mean a, standard deviation b.  Outliers are an independent Bernoulli(1e-3)
mask per entry; masked entries are multiplied by 50 before the bf16 cast.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

PER_SAMPLE = 0
PER_TOKEN = 1

VARLEN_CHOICES = (1560, 8190, 16380, 32760)
VARLEN_WEIGHTS = (0.5, 0.2, 0.2, 0.1)


@dataclass(frozen=True)
class Workload:
    index: int
    name: str
    dtype: str                      # "bf16" or "f32": the I/O element type
    B: int                          # samples (or segments for varlen)
    S: int                          # tokens per sample (0 for varlen)
    D: int
    mod: int = PER_SAMPLE
    x_mean: float = 0.0
    x_std: float = 1.0
    outlier_p: float = 0.0
    outlier_mul: float = 1.0
    varlen: bool = False
    backward: bool = True
    seed: int = 0
    eps: float = 1e-6


WORKLOADS = (
    Workload(0, "tiny_fp32", "f32", 2, 256, 1536, seed=1001),
    Workload(1, "wan1.3b_fwd", "bf16", 1, 32760, 1536, backward=False, seed=1002),
    Workload(2, "wan14b_fwd_bwd", "bf16", 1, 75600, 5120, x_mean=0.5, x_std=2.0,
             outlier_p=1e-3, outlier_mul=50.0, seed=1003),
    Workload(3, "per_token", "bf16", 2, 32760, 5120, mod=PER_TOKEN, seed=1004),
    Workload(4, "varlen_packed", "bf16", 24, 0, 5120, varlen=True, seed=1005),
)


@dataclass
class Inputs:
    workload: Workload
    x: np.ndarray                   # [T, D] float32
    shift: np.ndarray               # [B, D] / [nseg, D] / [T, D] float32
    scale: np.ndarray
    dy: Optional[np.ndarray]        # [T, D] float32, None for forward-only workloads
    cu_seqlens: np.ndarray          # [nseg+1] int32 token offsets (uniform for fixed length)
    B: int
    S: int                          # tokens per sample; 0 when lengths differ
    D: int
    lengths: tuple = field(default_factory=tuple)
    length_seed: Optional[int] = None

    @property
    def T(self) -> int:
        return int(self.x.shape[0])


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """The 16-bit patterns of float32 values that are already exact bf16 numbers."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    if np.any(u & np.uint32(0xFFFF)):
        raise ValueError("values are not exact bf16 numbers")
    return (u >> np.uint32(16)).astype(np.uint16)


def varlen_lengths(nseg: int = 24, lo: int = 140_000, hi: int = 160_000,
                   choices=VARLEN_CHOICES, weights=VARLEN_WEIGHTS, max_seed: int = 10_000):
    """Draw nseg lengths i.i.d. with the stated weights; seeds 0,1,2,... are tried in order and
    the first draw whose total lies in [lo, hi] is taken.  Returns (lengths, seed)."""
    for seed in range(max_seed):
        rng = np.random.default_rng(seed)
        lens = rng.choice(np.asarray(choices, dtype=np.int64), size=nseg, p=weights)
        if lo <= int(lens.sum()) <= hi:
            return tuple(int(v) for v in lens), seed
    raise RuntimeError("no seed below %d gives a total in [%d, %d]" % (max_seed, lo, hi))


def _normal(rng, shape, mean, std):
    a = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if mean != 0.0:
        a += np.float32(mean)
    return a


def make_inputs(index: int, *, S: Optional[int] = None, B: Optional[int] = None,
                D: Optional[int] = None, lengths=None, dtype: Optional[str] = None,
                seed: Optional[int] = None, with_dy: Optional[bool] = None) -> Inputs:
    """Inputs of workload `index`.  S, B, D, lengths, dtype and seed override the recipe's own
    values (smaller shapes of the same distribution for tests the CPU reference finishes
    quickly)."""
    w = WORKLOADS[index]
    B = w.B if B is None else int(B)
    D = w.D if D is None else int(D)
    dt = w.dtype if dtype is None else dtype
    rng = np.random.default_rng(w.seed if seed is None else seed)
    length_seed = None
    if w.varlen:
        if lengths is None:
            lengths, length_seed = varlen_lengths(B)
        lengths = tuple(int(v) for v in lengths)
        B = len(lengths)
        S_out = 0
    else:
        S_out = w.S if S is None else int(S)
        lengths = (S_out,) * B
    cu = np.zeros(B + 1, dtype=np.int64)
    np.cumsum(np.asarray(lengths, dtype=np.int64), out=cu[1:])
    T = int(cu[-1])
    if T >= 2 ** 31:
        raise ValueError("token count does not fit int32 offsets")

    x = _normal(rng, (T, D), w.x_mean, w.x_std)
    if w.outlier_p > 0.0:
        mask = rng.random((T, D), dtype=np.float32) < np.float32(w.outlier_p)
        x[mask] *= np.float32(w.outlier_mul)
        del mask
    mod_rows = T if w.mod == PER_TOKEN else B
    shift = _normal(rng, (mod_rows, D), 0.0, 0.1)
    scale = _normal(rng, (mod_rows, D), 0.0, 0.1)
    want_dy = w.backward if with_dy is None else with_dy
    dy = _normal(rng, (T, D), 0.0, 1.0) if want_dy else None
    if dt == "bf16":
        x = round_to_bf16(x)
        shift = round_to_bf16(shift)
        scale = round_to_bf16(scale)
        if dy is not None:
            dy = round_to_bf16(dy)
    elif dt != "f32":
        raise ValueError("dtype must be 'bf16' or 'f32'")
    w_out = Workload(**{**w.__dict__, "dtype": dt, "B": B, "S": S_out, "D": D})
    return Inputs(w_out, x, shift, scale, dy, cu.astype(np.int32), B, S_out, D,
                  lengths=lengths, length_seed=length_seed)


@dataclass
class GatedExtras:
    """The additional inputs of the gated residual + LayerNorm-Modulate operator."""
    u: np.ndarray                   # [T, D] branch output
    gate: np.ndarray                # [B, D] / [nseg, D]
    dh: np.ndarray                  # [T, D] gradient arriving along the residual stream


def make_gated_extras(inp: Inputs, seed: int) -> GatedExtras:
    """u ~ N(0, 1), gate ~ N(0, 0.3), dh ~ N(0, 1) for the token layout of `inp`, rounded to bf16
    when the workload's I/O type is bf16."""
    rng = np.random.default_rng(seed)
    T, D = inp.x.shape
    u = _normal(rng, (T, D), 0.0, 1.0)
    gate = _normal(rng, (inp.B, D), 0.0, 0.3)
    dh = _normal(rng, (T, D), 0.0, 1.0)
    if inp.workload.dtype == "bf16":
        u, gate, dh = round_to_bf16(u), round_to_bf16(gate), round_to_bf16(dh)
    return GatedExtras(u, gate, dh)


@dataclass
class QkNormInputs:
    """Inputs of the fused Q-Norm + K-Norm operator: float32 host arrays, exact in `dtype`."""
    q: np.ndarray                   # [N, D]
    k: np.ndarray
    wq: np.ndarray                  # [D]
    wk: np.ndarray
    dq_out: np.ndarray              # [N, D] gradients of the normalised tensors
    dk_out: np.ndarray
    dtype: str
    eps: float = 1e-6


def make_qknorm_inputs(N: int, D: int, dtype: str = "bf16", seed: int = 0,
                       outlier_p: float = 1e-3) -> QkNormInputs:
    """q ~ N(0, 1) and k ~ N(0.2, 2) with a Bernoulli(outlier_p) mask of entries multiplied by 30
    (projection outputs have heavy tails), weights ~ N(1, 0.1), upstream gradients ~ N(0, 1)."""
    rng = np.random.default_rng(seed)
    q = _normal(rng, (N, D), 0.0, 1.0)
    k = _normal(rng, (N, D), 0.2, 2.0)
    if outlier_p > 0.0 and N > 0:
        for a in (q, k):
            mask = rng.random((N, D), dtype=np.float32) < np.float32(outlier_p)
            a[mask] *= np.float32(30.0)
    wq, wk = _normal(rng, (D,), 1.0, 0.1), _normal(rng, (D,), 1.0, 0.1)
    dq, dk = _normal(rng, (N, D), 0.0, 1.0), _normal(rng, (N, D), 0.0, 1.0)
    arrs = [q, k, wq, wk, dq, dk]
    if dtype == "bf16":
        arrs = [round_to_bf16(a) for a in arrs]
    elif dtype != "f32":
        raise ValueError("dtype must be 'bf16' or 'f32'")
    return QkNormInputs(*arrs, dtype=dtype)
