"""MI355X-native fused LayerNorm-Modulate (AdaLN): hand-written gfx950 kernels behind a C ABI.

`lnmod` is the thin binding over the shared library (argument marshalling only);
`functional` wraps the three operators as torch.autograd functions;
`synth` holds the seeded synthetic workloads.
"""
from . import synth  # noqa: F401
