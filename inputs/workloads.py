"""The synthetic workloads: shapes, windows and seeds.

Each entry stands in for a serving workload of the model whose shape it takes
(Llama-3.1-8B: 32 layers, 32 query / 8 KV heads; Qwen2.5-7B: 28 layers, 28 query / 4 KV
heads; head_dim 128) with sink + recent windows in the range the paper ablates.  No
dataset or model content is involved: K, V and Q are seeded N(0,1) values, the first
four key positions of every head are scaled by 4 to mimic attention-sink tokens.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

from . import synth


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str            # "f32" | "bf16"
    batch: int
    ctx_lo: int           # context length range before the first decode step
    ctx_hi: int
    pct_compressed: int   # per-layer percentage of KV heads that are compressed
    sink: int
    recent: int
    decode_steps: int
    seed: int
    q_prescaled: bool = False      # Q already carries 1/sqrt(D); softmax_scale = 1
    sink_key_scale: float = 4.0
    n_sink_keys: int = 4
    fixed_mask: tuple | None = None  # per KV head, same for all layers (config 1)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def softmax_scale(self) -> float:
        return 1.0 if self.q_prescaled else 1.0 / float(np.sqrt(self.head_dim))

    def lengths(self) -> list[int]:
        return synth.ragged_lengths(self.seed, self.batch, self.ctx_lo, self.ctx_hi)

    def mask(self) -> np.ndarray:
        if self.fixed_mask is not None:
            return np.tile(np.asarray(self.fixed_mask, dtype=np.uint8), (self.n_layers, 1))
        return synth.head_mask(self.seed, self.n_layers, self.n_kv_heads, self.pct_compressed)

    def with_pct(self, pct: int) -> "Workload":
        return replace(self, pct_compressed=pct, fixed_mask=None,
                       name=f"{self.name.split('@')[0]}@{pct}")

    def all_full(self) -> "Workload":
        return replace(self, pct_compressed=0, fixed_mask=None, name=f"{self.name.split('@')[0]}@allfull")


_S = synth.BASE_SEED

WORKLOADS = {
    # single layer, fp32, heads 0-3 full / 4-7 compressed, Q pre-scaled by 1/sqrt(128)
    "c1": Workload("c1", 1, 32, 8, 128, "f32", 1, 1024, 1024, 50, 16, 112, 16, _S + 1,
                   q_prescaled=True, sink_key_scale=1.0, n_sink_keys=0,
                   fixed_mask=(1, 1, 1, 1, 0, 0, 0, 0)),
    "c2": Workload("c2", 32, 32, 8, 128, "bf16", 8, 8192, 8192, 20, 64, 256, 16, _S + 2),
    "c3": Workload("c3", 28, 28, 4, 128, "bf16", 16, 16384, 16384, 60, 64, 256, 16, _S + 3),
    "c4": Workload("c4", 32, 32, 8, 128, "bf16", 32, 4096, 32768, 60, 64, 512, 128, _S + 4),
    "c5": Workload("c5", 32, 32, 8, 128, "bf16", 64, 16384, 65536, 60, 64, 256, 512, _S + 5),
}


def algorithmic_bytes_per_step(w: Workload, lengths_after_append, mask: np.ndarray) -> int:
    """Bytes the method itself must move for one decode step over all layers.

    KV rows of every head's effective history (full: n, compressed: min(n, sink+recent)),
    K and V, plus the query read, the output write and the appended K/V rows.
    """
    e = 4 if w.dtype == "f32" else 2
    D = w.head_dim
    W = w.sink + w.recent
    total = 0
    n_arr = np.asarray(lengths_after_append, dtype=np.int64)
    n_comp = np.minimum(n_arr, W)
    for l in range(w.n_layers):
        n_full_heads = int(mask[l].sum())
        n_comp_heads = w.n_kv_heads - n_full_heads
        total += 2 * D * e * int(n_full_heads * n_arr.sum() + n_comp_heads * n_comp.sum())
    total += w.n_layers * w.batch * (2 * w.n_q_heads * D * e + 2 * w.n_kv_heads * D * e)
    return int(total)
