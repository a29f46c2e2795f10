"""CPU oracle (test infrastructure only; never imported by the product package)."""
from .oracle import (build, decode_attention, decode_attention_gated, in_position_set, num_threads, prefill_attention,  # noqa: F401
                     ring_simulate)
