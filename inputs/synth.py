"""Seeded synthetic inputs for head-mixed KV-cache decode attention.

This module only makes numbers: a counter-based generator whose every value is a pure
function of (seed, tensor id, layer, sequence, head, position, dim), plus the seeded
choices a workload needs (ragged context lengths, per-layer full/compressed head mask).
It holds none of the attention / cache arithmetic and is the one module that both the
CPU oracle's tests and the HIP path's tests and benchmark may import.

All hashing is integer arithmetic on int64 tensors whose values stay below 2**32 and
whose products stay below 2**63, so the CPU and the GPU (same torch ops, other device)
produce bit-identical results.  Normal variates come from a 65 536-entry inverse-CDF
table built once on the host in float64 and looked up by a 16-bit hash, so no
transcendental function is evaluated on the device.
"""
from __future__ import annotations

import functools
from typing import Sequence

import numpy as np
import torch

BASE_SEED = 251008525

# tensor ids
T_K, T_V, T_Q, T_LEN, T_SCORE = 1, 2, 3, 4, 5

_M32 = 0xFFFFFFFF
_MUL = 0x45D9F3B  # < 2**27, so (x < 2**32) * _MUL < 2**59: no int64 overflow


def _mix_int(x: int) -> int:
    """32-bit avalanche mix of a Python int (same steps as _mix_t)."""
    x &= _M32
    x ^= x >> 16
    x = (x * _MUL) & _M32
    x ^= x >> 16
    x = (x * _MUL) & _M32
    x ^= x >> 16
    return x


def _mix_t(x: torch.Tensor) -> torch.Tensor:
    """32-bit avalanche mix of an int64 tensor with values in [0, 2**32)."""
    x = x ^ (x >> 16)
    x = (x * _MUL) & _M32
    x = x ^ (x >> 16)
    x = (x * _MUL) & _M32
    x = x ^ (x >> 16)
    return x


def _keys(seed: int, tensor_id: int, layer: int, seqs: torch.Tensor, heads: torch.Tensor):
    """Two 32-bit stream keys per (seq, head): int64 tensors of shape [nseq, nhead]."""
    base = _mix_int(_mix_int(seed) + 0x9E3779B1 * (tensor_id + 1))
    base = _mix_int(base + 0x85EBCA77 * (layer + 1))
    s = _mix_t((seqs.to(torch.int64)[:, None] * 0x27D4EB2F + base) & _M32)
    a = _mix_t((s + heads.to(torch.int64)[None, :] * 0x165667B1 + 1) & _M32)
    b = _mix_t(((a ^ 0x5BD1E995) + 0x1B873593) & _M32)
    return a, b


@functools.lru_cache(maxsize=None)
def _icdf_table_host() -> torch.Tensor:
    from scipy.special import ndtri

    p = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
    return torch.from_numpy(ndtri(p).astype(np.float32))


_table_cache: dict = {}


def icdf_table(device) -> torch.Tensor:
    """float32 [65536] standard-normal quantiles at the bin centres, on `device`."""
    key = str(device)
    if key not in _table_cache:
        _table_cache[key] = _icdf_table_host().to(device)
    return _table_cache[key]


def hash_u32_at(seed: int, tensor_id: int, layer: int, seqs, heads, pos: torch.Tensor, dim: int,
                device="cpu") -> torch.Tensor:
    """Raw 32-bit hashes at per-sequence positions pos [nseq, npos]: int64 [nseq, nhead, npos, dim]."""
    seqs = torch.as_tensor(seqs, dtype=torch.int64, device=device).reshape(-1)
    heads = torch.as_tensor(heads, dtype=torch.int64, device=device).reshape(-1)
    ka, kb = _keys(seed, tensor_id, layer, seqs, heads)
    pos = torch.as_tensor(pos, dtype=torch.int64, device=device)
    d = torch.arange(dim, dtype=torch.int64, device=device)
    idx = (pos[:, None, :, None] * dim + d[None, None, None, :]) & _M32    # [nseq, 1, npos, dim]
    x = _mix_t(idx ^ ka[:, :, None, None])
    x = _mix_t((x + kb[:, :, None, None]) & _M32)
    return x


def hash_u32(seed: int, tensor_id: int, layer: int, seqs, heads, pos0: int, npos: int,
             dim: int, device="cpu") -> torch.Tensor:
    """Raw 32-bit hashes of positions pos0..pos0+npos-1, int64 [nseq, nhead, npos, dim]."""
    nseq = len(seqs) if not torch.is_tensor(seqs) else seqs.numel()
    pos = torch.arange(pos0, pos0 + npos, dtype=torch.int64, device=device)[None, :].expand(nseq, npos)
    return hash_u32_at(seed, tensor_id, layer, seqs, heads, pos, dim, device)


def normal_at(seed: int, tensor_id: int, layer: int, seqs, heads, pos, dim: int, dtype=torch.float32,
              device="cpu", sink_scale: float = 1.0, n_sink_scaled: int = 0) -> torch.Tensor:
    """N(0,1) values [nseq, nhead, npos, dim] at per-sequence positions pos [nseq, npos].

    Positions < n_sink_scaled are multiplied by `sink_scale` before rounding to `dtype`
    (the "attention-sink keys" of the workload recipe).
    """
    pos = torch.as_tensor(pos, dtype=torch.int64, device=device)
    x = hash_u32_at(seed, tensor_id, layer, seqs, heads, pos, dim, device)
    vals = icdf_table(device)[(x >> 16)]
    if n_sink_scaled > 0 and sink_scale != 1.0:
        factor = torch.where(pos < n_sink_scaled, sink_scale, 1.0).to(vals.dtype)
        vals = vals * factor[:, None, :, None]
    return vals.to(dtype)


def normal(seed: int, tensor_id: int, layer: int, seqs, heads, pos0: int, npos: int,
           dim: int, dtype=torch.float32, device="cpu", sink_scale: float = 1.0,
           n_sink_scaled: int = 0) -> torch.Tensor:
    """N(0,1) values [nseq, nhead, npos, dim] at positions pos0..pos0+npos-1 (see normal_at)."""
    nseq = len(seqs) if not torch.is_tensor(seqs) else seqs.numel()
    pos = torch.arange(pos0, pos0 + npos, dtype=torch.int64, device=device)[None, :].expand(nseq, npos)
    return normal_at(seed, tensor_id, layer, seqs, heads, pos, dim, dtype, device, sink_scale, n_sink_scaled)


def ragged_lengths(seed: int, batch: int, lo: int, hi: int) -> list[int]:
    """Per-sequence context lengths, uniform on [lo, hi] by hash (lo == hi: constant)."""
    out = []
    base = _mix_int(_mix_int(seed) + 0x9E3779B1 * (T_LEN + 1))
    for b in range(batch):
        h = _mix_int(_mix_int(base + 0x27D4EB2F * b) + 0x165667B1)
        out.append(lo + h % (hi - lo + 1))
    return out


def head_scores(seed: int, n_layers: int, n_kv_heads: int) -> np.ndarray:
    """Seeded stand-in for per-(layer, KV head) importance scores: uint32 [L, Hkv]."""
    base = _mix_int(_mix_int(seed) + 0x9E3779B1 * (T_SCORE + 1))
    sc = np.zeros((n_layers, n_kv_heads), dtype=np.uint32)
    for l in range(n_layers):
        for h in range(n_kv_heads):
            sc[l, h] = _mix_int(_mix_int(base + 0x85EBCA77 * (l + 1)) + 0x165667B1 * h + 1)
    return sc


def head_mask(seed: int, n_layers: int, n_kv_heads: int, pct_compressed: int) -> np.ndarray:
    """uint8 [L, Hkv], 1 = full history, 0 = compressed (sink + recent).

    Per layer the lowest-scoring heads are compressed.  The per-layer count follows an
    integer error-diffusion so that fractional head counts average to the requested
    percentage: count(l) = floor((l+1)*pct*Hkv/100) - floor(l*pct*Hkv/100).  Ties are
    broken towards the lower head index.
    """
    sc = head_scores(seed, n_layers, n_kv_heads)
    mask = np.ones((n_layers, n_kv_heads), dtype=np.uint8)
    for l in range(n_layers):
        cnt = ((l + 1) * pct_compressed * n_kv_heads) // 100 - (l * pct_compressed * n_kv_heads) // 100
        order = sorted(range(n_kv_heads), key=lambda h: (int(sc[l, h]), h))
        for h in order[:cnt]:
            mask[l, h] = 0
    return mask


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """Bit pattern of a CPU bf16 tensor as a uint16 numpy array (same shape)."""
    assert t.dtype == torch.bfloat16 and t.device.type == "cpu"
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)
