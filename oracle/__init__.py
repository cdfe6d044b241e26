"""float64 CPU oracles of the LayerNorm-Modulate operator (lnmod_oracle) and of its
gated-residual variant (gated_oracle) and of the fused Q-Norm + K-Norm (qknorm_oracle): test
infrastructure, not product."""
from .lnmod_oracle import (PER_SEGMENT, PER_TOKEN, backward, build, forward, load,  # noqa: F401
                           num_threads, set_num_threads)
