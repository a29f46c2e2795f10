"""ctypes front end of the C oracle (oracle/rlkv_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's
cpu_baseline leg.  Nothing here touches the HIP library or shares code with it.
Arrays are numpy; bf16 tensors are passed as their uint16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rlkv_oracle.c")
_LIB = os.path.join(_HERE, "librlkv_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over independent outputs)."""
    deps = [_SRC, os.path.join(_HERE, "attend_body.inc")]
    stale = (not os.path.exists(_LIB)) or any(os.path.getmtime(d) > os.path.getmtime(_LIB) for d in deps)
    if force or stale:
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"], cwd=_HERE)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, i32, i64, dbl = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_double
        for name in ("rlkv_oracle_decode_f64", "rlkv_oracle_decode_f32"):
            f = getattr(lib, name)
            f.restype = i32
            f.argtypes = [i32, vp, vp, i64, vp, vp, i32, i32, i32, i32, i32, i32, dbl, vp, vp, vp]
        for name in ("rlkv_oracle_decode_gated_f64", "rlkv_oracle_decode_gated_f32"):
            f = getattr(lib, name)
            f.restype = i32
            f.argtypes = [i32, vp, vp, i64, vp, vp, i32, i32, i32, i32, i32, i32, dbl, vp, vp]
        for name in ("rlkv_oracle_prefill_f64", "rlkv_oracle_prefill_f32"):
            f = getattr(lib, name)
            f.restype = i32
            f.argtypes = [i32, vp, vp, i64, vp, vp, i32, vp, i32, i32, i32, i32, i32, i32, dbl, vp, vp]
        lib.rlkv_oracle_in_position_set.restype = i32
        lib.rlkv_oracle_in_position_set.argtypes = [i32, i64, i64, i32, i32]
        lib.rlkv_oracle_ring_simulate.restype = i64
        lib.rlkv_oracle_ring_simulate.argtypes = [i32, i32, i64, vp]
        lib.rlkv_oracle_num_threads.restype = i32
        _lib = lib
    return _lib


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    raise TypeError(f"oracle takes float32 or bf16-as-uint16 arrays, got {a.dtype}")


def decode_attention(k_hist: np.ndarray, v_hist: np.ndarray, n, full_mask, q: np.ndarray,
                     sink: int, recent: int, scale: float, precision: str = "f64",
                     return_weights: bool = False):
    """One layer of decode attention from the complete history.

    k_hist, v_hist: [B, Hkv, cap, D] (float32 or uint16 bf16 bits); n: [B] lengths;
    full_mask: [Hkv]; q: [B, Hq, D] same dtype.  Returns out [B, Hq, D] (float64 or
    float32 per `precision`), and the weights [B, Hq, cap] if asked.
    """
    lib = _load()
    k_hist = np.ascontiguousarray(k_hist)
    v_hist = np.ascontiguousarray(v_hist)
    q = np.ascontiguousarray(q)
    code = _dtype_code(k_hist)
    assert _dtype_code(v_hist) == code and _dtype_code(q) == code
    B, Hkv, cap, D = k_hist.shape
    assert v_hist.shape == k_hist.shape
    Bq, Hq, Dq = q.shape
    assert Bq == B and Dq == D
    n = np.ascontiguousarray(np.asarray(n, dtype=np.int32).reshape(B))
    full_mask = np.ascontiguousarray(np.asarray(full_mask, dtype=np.uint8).reshape(Hkv))
    real = np.float64 if precision == "f64" else np.float32
    out = np.empty((B, Hq, D), dtype=real)
    weights = np.empty((B, Hq, cap), dtype=real) if return_weights else None
    fn = lib.rlkv_oracle_decode_f64 if precision == "f64" else lib.rlkv_oracle_decode_f32
    rc = fn(code, k_hist.ctypes.data, v_hist.ctypes.data, cap, n.ctypes.data,
            full_mask.ctypes.data, B, Hq, Hkv, D, int(sink), int(recent), float(scale),
            q.ctypes.data, out.ctypes.data, weights.ctypes.data if weights is not None else None)
    if rc != 0:
        raise ValueError("oracle: invalid argument")
    return (out, weights) if return_weights else out


def decode_attention_gated(k_hist: np.ndarray, v_hist: np.ndarray, n, gate, q: np.ndarray, sink: int,
                           recent: int, scale: float, precision: str = "f64"):
    """Eq. 1: gate[h] * full attention + (1 - gate[h]) * local attention, complete history for
    every head.  Shapes as in decode_attention; gate: [Hkv] in [0, 1]."""
    lib = _load()
    k_hist = np.ascontiguousarray(k_hist)
    v_hist = np.ascontiguousarray(v_hist)
    q = np.ascontiguousarray(q)
    code = _dtype_code(k_hist)
    assert _dtype_code(v_hist) == code and _dtype_code(q) == code
    B, Hkv, cap, D = k_hist.shape
    Bq, Hq, Dq = q.shape
    assert v_hist.shape == k_hist.shape and Bq == B and Dq == D
    n = np.ascontiguousarray(np.asarray(n, dtype=np.int32).reshape(B))
    gate = np.ascontiguousarray(np.asarray(gate, dtype=np.float64).reshape(Hkv))
    real = np.float64 if precision == "f64" else np.float32
    out = np.empty((B, Hq, D), dtype=real)
    fn = lib.rlkv_oracle_decode_gated_f64 if precision == "f64" else lib.rlkv_oracle_decode_gated_f32
    rc = fn(code, k_hist.ctypes.data, v_hist.ctypes.data, cap, n.ctypes.data, gate.ctypes.data, B, Hq, Hkv, D,
            int(sink), int(recent), float(scale), q.ctypes.data, out.ctypes.data)
    if rc != 0:
        raise ValueError("oracle: invalid argument")
    return out


def prefill_attention(k_hist: np.ndarray, v_hist: np.ndarray, n_old, t, gate, q: np.ndarray, sink: int,
                      recent: int, scale: float, precision: str = "f64"):
    """Prefill (one chunk) with mixed heads: row c of sequence b is the query at position
    n_old[b] + c; gate[h] = 1 -> causal mask, 0 -> local mask (sink + recent), between -> Eq. 1 blend.

    k_hist, v_hist: [B, Hkv, cap, D] complete history including the chunk; q: [B, Hq, T, D];
    n_old, t: [B].  Returns out [B, Hq, T, D]; rows c >= t[b] are NaN."""
    lib = _load()
    k_hist = np.ascontiguousarray(k_hist)
    v_hist = np.ascontiguousarray(v_hist)
    q = np.ascontiguousarray(q)
    code = _dtype_code(k_hist)
    assert _dtype_code(v_hist) == code and _dtype_code(q) == code
    B, Hkv, cap, D = k_hist.shape
    Bq, Hq, T, Dq = q.shape
    assert v_hist.shape == k_hist.shape and Bq == B and Dq == D
    n_old = np.ascontiguousarray(np.asarray(n_old, dtype=np.int32).reshape(B))
    t = np.ascontiguousarray(np.asarray(t, dtype=np.int32).reshape(B))
    gate = np.ascontiguousarray(np.asarray(gate, dtype=np.float64).reshape(Hkv))
    real = np.float64 if precision == "f64" else np.float32
    out = np.full((B, Hq, T, D), np.nan, dtype=real)
    fn = lib.rlkv_oracle_prefill_f64 if precision == "f64" else lib.rlkv_oracle_prefill_f32
    rc = fn(code, k_hist.ctypes.data, v_hist.ctypes.data, cap, n_old.ctypes.data, t.ctypes.data, T,
            gate.ctypes.data, B, Hq, Hkv, D, int(sink), int(recent), float(scale), q.ctypes.data, out.ctypes.data)
    if rc != 0:
        raise ValueError("oracle: invalid argument")
    return out


def in_position_set(is_full: bool, j: int, n: int, sink: int, recent: int) -> bool:
    return bool(_load().rlkv_oracle_in_position_set(int(is_full), j, n, sink, recent))


def ring_simulate(sink: int, recent: int, n_tokens: int):
    """(slot_pos [sink+recent] int32, cached length) after n_tokens one-token appends."""
    lib = _load()
    slot_pos = np.empty(sink + recent, dtype=np.int32)
    length = lib.rlkv_oracle_ring_simulate(sink, recent, n_tokens, slot_pos.ctypes.data)
    return slot_pos, int(length)


def num_threads() -> int:
    return int(_load().rlkv_oracle_num_threads())
