"""CPU oracle (test infrastructure only; never imported by the product package)."""
from .oracle import (build, decode_attention, decode_attention_gated, in_position_set, num_threads,  # noqa: F401
                     ring_simulate)
