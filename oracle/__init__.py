"""float64 CPU oracle of the LayerNorm-Modulate operator: test infrastructure, not product."""
from .lnmod_oracle import (PER_SEGMENT, PER_TOKEN, backward, build, forward, load,  # noqa: F401
                           num_threads, set_num_threads)
