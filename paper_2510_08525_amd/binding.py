"""ctypes binding of librlkv.so: the same names as include/rlkv.h, marshalling only.

Every step of the hot path runs inside the library's HIP kernels.  There is no Python or
CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "librlkv.so")
_lib = None

RLKV_OK, RLKV_ERR_INVALID_ARG, RLKV_ERR_OOM, RLKV_ERR_CAPACITY, RLKV_ERR_STATE, RLKV_ERR_HIP, RLKV_ERR_TOO_LARGE = range(7)
RLKV_F32, RLKV_BF16 = 0, 1
RLKV_KERNEL_AUTO, RLKV_KERNEL_VALU, RLKV_KERNEL_MFMA = 0, 1, 2


class RlkvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {rlkv_status_string(status)} (status {status})")


class _Config(ctypes.Structure):
    _fields_ = [
        ("n_layers", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("batch", ctypes.c_int32), ("sink", ctypes.c_int32),
        ("recent", ctypes.c_int32), ("dtype", ctypes.c_int32), ("kernel", ctypes.c_int32),
        ("device", ctypes.c_int32), ("full_mask", ctypes.c_void_p), ("max_len", ctypes.c_void_p),
        ("arena", ctypes.c_void_p), ("arena_bytes", ctypes.c_size_t),
        ("page_tokens", ctypes.c_int32), ("pool_pages", ctypes.c_int32), ("prefill_tokens", ctypes.c_int32),
        ("decode_wgs_per_cu", ctypes.c_int32), ("prefill_min_share_tiles", ctypes.c_int32),
        ("prefill_two_group_only", ctypes.c_int32),
    ]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads librlkv.so built in-tree (python -m paper_2510_08525_amd.build); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is not built: run `python -m paper_2510_08525_amd.build` "
                          "(there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, sz, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t, ctypes.c_float
    cfgp = ctypes.POINTER(_Config)
    sigs = {
        "rlkv_cache_required_bytes": (sz, [cfgp]),
        "rlkv_cache_create": (i32, [cfgp, ctypes.POINTER(vp)]),
        "rlkv_cache_destroy": (i32, [vp]),
        "rlkv_cache_reset": (i32, [vp, i32, vp]),
        "rlkv_append": (i32, [vp, i32, vp, vp, i32, vp]),
        "rlkv_append_ragged": (i32, [vp, i32, vp, vp, vp, i32, vp]),
        "rlkv_decode_attention": (i32, [vp, i32, vp, vp, f32, vp]),
        "rlkv_decode_attention_noalloc": (i32, [vp, i32, vp, vp, f32, vp]),
        "rlkv_set_active": (i32, [vp, vp, vp]),
        "rlkv_set_gates": (i32, [vp, vp, vp]),
        "rlkv_append_decode": (i32, [vp, i32, vp, vp, vp, vp, f32, vp]),
        "rlkv_append_decode_prepare": (i32, [vp, i32, vp]),
        "rlkv_append_decode_launch": (i32, [vp, i32, vp, vp, vp, vp, f32, vp]),
        "rlkv_worklists_built": (ctypes.c_int64, [vp]),
        "rlkv_prefill_attention": (i32, [vp, i32, vp, vp, vp, vp, i32, vp, f32, vp]),
        "rlkv_profile_enable": (i32, [vp, i32]),
        "rlkv_profile_collect": (i32, [vp, vp, vp]),
        "rlkv_get_lengths": (i32, [vp, i32, vp]),
        "rlkv_get_slot_positions": (i32, [vp, i32, i32, i32, vp]),
        "rlkv_resident_bytes": (sz, [vp]),
        "rlkv_probe_stream_read": (i32, [vp, sz, vp, i32, vp]),
        "rlkv_plan_shares": (i32, [vp, i32, i32, vp, vp, vp]),
        "rlkv_plan_prefill_form": (i32, [i32, i32, i32, i32, i32, vp, vp, i32, i32, vp, vp]),
        "rlkv_plan_prefill_rows": (i32, [i32, i32, vp, vp, vp, vp]),
        "rlkv_plan_prefill_block": (i32, [i32, i32, i32, i32, i32, vp, vp]),
        "rlkv_cache_kernel": (i32, [vp]),
        "rlkv_pool_pages_free": (ctypes.c_int64, [vp]),
        "rlkv_pool_shuffle": (i32, [vp, ctypes.c_uint64]),
        "rlkv_status_string": (ctypes.c_char_p, [i32]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


EXPORTED_SYMBOLS = (
    "rlkv_cache_required_bytes", "rlkv_cache_create", "rlkv_cache_destroy", "rlkv_cache_reset",
    "rlkv_append", "rlkv_append_ragged", "rlkv_decode_attention", "rlkv_decode_attention_noalloc", "rlkv_set_active", "rlkv_set_gates", "rlkv_append_decode", "rlkv_append_decode_prepare", "rlkv_append_decode_launch", "rlkv_worklists_built", "rlkv_prefill_attention", "rlkv_profile_enable",
    "rlkv_profile_collect", "rlkv_get_lengths",
    "rlkv_get_slot_positions", "rlkv_resident_bytes", "rlkv_probe_stream_read", "rlkv_plan_shares", "rlkv_plan_prefill_form", "rlkv_plan_prefill_rows", "rlkv_plan_prefill_block", "rlkv_cache_kernel", "rlkv_pool_pages_free",
    "rlkv_pool_shuffle", "rlkv_status_string",
)


def rlkv_status_string(status: int) -> str:
    return load_library().rlkv_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != RLKV_OK:
        raise RlkvError(status, where)


def _make_config(n_layers, n_q_heads, n_kv_heads, head_dim, batch, sink, recent, dtype, full_mask,
                 max_len, kernel=RLKV_KERNEL_AUTO, device=0, arena_ptr=0, arena_bytes=0, page_tokens=0,
                 pool_pages=0, prefill_tokens=0, decode_wgs_per_cu=0, prefill_min_share_tiles=0,
                 prefill_two_group_only=0):
    """Returns (config struct, keep-alive objects)."""
    mask = None if full_mask is None else np.ascontiguousarray(np.asarray(full_mask, dtype=np.uint8).reshape(-1))
    mlen = None if max_len is None else np.ascontiguousarray(np.asarray(max_len, dtype=np.int32).reshape(-1))
    if mask is not None and n_layers > 0 and n_kv_heads > 0 and mask.size != n_layers * n_kv_heads:
        raise ValueError("full_mask must have n_layers * n_kv_heads entries")
    if mlen is not None and batch > 0 and mlen.size != batch:
        raise ValueError("max_len must have batch entries")
    cfg = _Config(n_layers, n_q_heads, n_kv_heads, head_dim, batch, sink, recent, dtype, kernel, device,
                  mask.ctypes.data if mask is not None else None,
                  mlen.ctypes.data if mlen is not None else None,
                  arena_ptr or None, arena_bytes, page_tokens, pool_pages, prefill_tokens, decode_wgs_per_cu,
                  prefill_min_share_tiles, prefill_two_group_only)
    return cfg, (mask, mlen)


def rlkv_cache_required_bytes(**kw) -> int:
    cfg, _keep = _make_config(**kw)
    return int(load_library().rlkv_cache_required_bytes(ctypes.byref(cfg)))


def rlkv_cache_create(**kw) -> int:
    """Returns the opaque cache handle (an integer address)."""
    cfg, _keep = _make_config(**kw)
    handle = ctypes.c_void_p()
    _check(load_library().rlkv_cache_create(ctypes.byref(cfg), ctypes.byref(handle)), "rlkv_cache_create")
    return handle.value


def rlkv_cache_destroy(handle: int):
    _check(load_library().rlkv_cache_destroy(handle), "rlkv_cache_destroy")


def rlkv_cache_reset(handle: int, seq: int = -1, stream: int = 0):
    _check(load_library().rlkv_cache_reset(handle, seq, stream or None), "rlkv_cache_reset")


def rlkv_append(handle: int, layer: int, k_ptr: int, v_ptr: int, n_tokens: int, stream: int = 0):
    _check(load_library().rlkv_append(handle, layer, k_ptr or None, v_ptr or None, n_tokens, stream or None),
           "rlkv_append")


def rlkv_append_ragged(handle: int, layer: int, k_ptr: int, v_ptr: int, n_tokens: Sequence[int],
                       stride_tokens: int, stream: int = 0):
    cnt = np.ascontiguousarray(np.asarray(n_tokens, dtype=np.int32))
    _check(load_library().rlkv_append_ragged(handle, layer, k_ptr or None, v_ptr or None, cnt.ctypes.data,
                                             stride_tokens, stream or None), "rlkv_append_ragged")


def rlkv_decode_attention(handle: int, layer: int, q_ptr: int, out_ptr: int, softmax_scale: float,
                          stream: int = 0):
    _check(load_library().rlkv_decode_attention(handle, layer, q_ptr or None, out_ptr or None,
                                                float(softmax_scale), stream or None), "rlkv_decode_attention")


def rlkv_decode_attention_noalloc(handle: int, layer: int, q_ptr: int, out_ptr: int, softmax_scale: float,
                                  stream: int = 0):
    _check(load_library().rlkv_decode_attention_noalloc(handle, layer, q_ptr or None, out_ptr or None,
                                                        float(softmax_scale), stream or None),
           "rlkv_decode_attention_noalloc")


def rlkv_set_active(handle: int, active, stream: int = 0):
    arr = None if active is None else np.ascontiguousarray(np.asarray(active, dtype=np.uint8))
    _check(load_library().rlkv_set_active(handle, arr.ctypes.data if arr is not None else None, stream or None),
           "rlkv_set_active")


def rlkv_set_gates(handle: int, gates, stream: int = 0):
    arr = None if gates is None else np.ascontiguousarray(np.asarray(gates, dtype=np.float32).reshape(-1))
    _check(load_library().rlkv_set_gates(handle, arr.ctypes.data if arr is not None else None, stream or None),
           "rlkv_set_gates")


def rlkv_append_decode(handle: int, layer: int, k_ptr: int, v_ptr: int, q_ptr: int, out_ptr: int,
                       softmax_scale: float, stream: int = 0):
    _check(load_library().rlkv_append_decode(handle, layer, k_ptr or None, v_ptr or None, q_ptr or None,
                                             out_ptr or None, float(softmax_scale), stream or None),
           "rlkv_append_decode")


def rlkv_append_decode_prepare(handle: int, layer: int, stream: int = 0):
    _check(load_library().rlkv_append_decode_prepare(handle, layer, stream or None), "rlkv_append_decode_prepare")


def rlkv_append_decode_launch(handle: int, layer: int, k_ptr: int, v_ptr: int, q_ptr: int, out_ptr: int,
                              softmax_scale: float, stream: int = 0):
    _check(load_library().rlkv_append_decode_launch(handle, layer, k_ptr or None, v_ptr or None, q_ptr or None,
                                                    out_ptr or None, float(softmax_scale), stream or None),
           "rlkv_append_decode_launch")


def rlkv_worklists_built(handle: int) -> int:
    return int(load_library().rlkv_worklists_built(handle))


def rlkv_prefill_attention(handle: int, layer: int, q_ptr: int, k_ptr: int, v_ptr: int, n_tokens: Sequence[int],
                           stride_tokens: int, out_ptr: int, softmax_scale: float, stream: int = 0):
    cnt = np.ascontiguousarray(np.asarray(n_tokens, dtype=np.int32))
    _check(load_library().rlkv_prefill_attention(handle, layer, q_ptr or None, k_ptr or None, v_ptr or None,
                                                 cnt.ctypes.data, stride_tokens, out_ptr or None,
                                                 float(softmax_scale), stream or None), "rlkv_prefill_attention")


def rlkv_profile_enable(handle: int, max_records: int):
    _check(load_library().rlkv_profile_enable(handle, max_records), "rlkv_profile_enable")


def rlkv_profile_collect(handle: int, max_records: int) -> np.ndarray:
    ms = np.zeros(max_records, dtype=np.float32)
    n = ctypes.c_int32(0)
    _check(load_library().rlkv_profile_collect(handle, ms.ctypes.data, ctypes.byref(n)), "rlkv_profile_collect")
    return ms[:n.value].copy()


def rlkv_get_lengths(handle: int, layer: int, batch: int) -> np.ndarray:
    out = np.empty(batch, dtype=np.int32)
    _check(load_library().rlkv_get_lengths(handle, layer, out.ctypes.data), "rlkv_get_lengths")
    return out


def rlkv_get_slot_positions(handle: int, layer: int, kv_head: int, seq: int, window: int) -> np.ndarray:
    out = np.empty(window, dtype=np.int32)
    _check(load_library().rlkv_get_slot_positions(handle, layer, kv_head, seq, out.ctypes.data),
           "rlkv_get_slot_positions")
    return out


def rlkv_resident_bytes(handle: int) -> int:
    return int(load_library().rlkv_resident_bytes(handle))


def rlkv_probe_stream_read(buf_ptr: int, nbytes: int, sink_ptr: int, workgroups: int, stream: int = 0):
    _check(load_library().rlkv_probe_stream_read(buf_ptr or None, nbytes, sink_ptr or None, workgroups, stream or None),
           "rlkv_probe_stream_read")


def rlkv_plan_shares(rounds, n_workgroups: int):
    """Returns (workgroups used, wg_begin [n_workgroups + 1], seg_first [n_pairs], seg_count [n_pairs])."""
    r = np.ascontiguousarray(np.asarray(rounds, dtype=np.int32).reshape(-1))
    wg_begin = np.zeros(n_workgroups + 1, dtype=np.int32)
    seg_first = np.zeros(r.size, dtype=np.int32)
    seg_count = np.zeros(r.size, dtype=np.int32)
    used = load_library().rlkv_plan_shares(r.ctypes.data, r.size, n_workgroups, wg_begin.ctypes.data,
                                           seg_first.ctypes.data, seg_count.ctypes.data)
    if used < 0:
        raise RlkvError(RLKV_ERR_INVALID_ARG, "rlkv_plan_shares")
    return int(used), wg_begin, seg_first, seg_count


def rlkv_plan_prefill_form(n_compute_units: int, n_q_heads: int, n_kv_heads: int, n_full_heads: int, n_tokens, cached,
                           min_share_tiles: int = 80, allow_narrow: bool = True):
    """Returns (narrow, n_split): the kernel form and the shares per full-head workgroup of one prefill chunk."""
    t = np.ascontiguousarray(np.asarray(n_tokens, dtype=np.int32).reshape(-1))
    c = np.ascontiguousarray(np.asarray(cached, dtype=np.int32).reshape(-1))
    if t.size != c.size:
        raise RlkvError(RLKV_ERR_INVALID_ARG, "rlkv_plan_prefill_form")
    narrow = np.zeros(1, dtype=np.int32)
    n_split = np.zeros(1, dtype=np.int32)
    rc = load_library().rlkv_plan_prefill_form(n_compute_units, n_q_heads, n_kv_heads, n_full_heads, t.size, t.ctypes.data,
                                               c.ctypes.data, min_share_tiles, 1 if allow_narrow else 0,
                                               narrow.ctypes.data, n_split.ctypes.data)
    if rc != 0:
        raise RlkvError(RLKV_ERR_INVALID_ARG, "rlkv_plan_prefill_form")
    return bool(narrow[0]), int(n_split[0])


def rlkv_plan_prefill_rows(n_full_heads: int, n_tokens, cached):
    """Returns (dealt_rows, heavy_rows): the leading grid rows of a prefill chunk that go one row per XCD, and the
    rows of full heads of sequences that have a chunk."""
    t = np.ascontiguousarray(np.asarray(n_tokens, dtype=np.int32).reshape(-1))
    c = np.ascontiguousarray(np.asarray(cached, dtype=np.int32).reshape(-1))
    if t.size != c.size:
        raise RlkvError(RLKV_ERR_INVALID_ARG, "rlkv_plan_prefill_rows")
    dealt = np.zeros(1, dtype=np.int32)
    heavy = np.zeros(1, dtype=np.int32)
    rc = load_library().rlkv_plan_prefill_rows(n_full_heads, t.size, t.ctypes.data, c.ctypes.data, dealt.ctypes.data,
                                               heavy.ctypes.data)
    if rc != 0:
        raise RlkvError(RLKV_ERR_INVALID_ARG, "rlkv_plan_prefill_rows")
    return int(dealt[0]), int(heavy[0])


def rlkv_plan_prefill_block(linear_index: int, grid_x: int, grid_y: int, dealt_rows: int, heavy_rows: int):
    """Returns the (x, y) block of a prefill attention launch that the workgroup with this linear index works on."""
    bx = ctypes.c_int32(0)
    by = ctypes.c_int32(0)
    rc = load_library().rlkv_plan_prefill_block(linear_index, grid_x, grid_y, dealt_rows, heavy_rows,
                                                ctypes.addressof(bx), ctypes.addressof(by))
    if rc != 0:
        raise RlkvError(RLKV_ERR_INVALID_ARG, "rlkv_plan_prefill_block")
    return bx.value, by.value


def rlkv_cache_kernel(handle: int) -> int:
    return int(load_library().rlkv_cache_kernel(handle))


def rlkv_pool_pages_free(handle: int) -> int:
    return int(load_library().rlkv_pool_pages_free(handle))


def rlkv_pool_shuffle(handle: int, seed: int):
    _check(load_library().rlkv_pool_shuffle(handle, ctypes.c_uint64(seed)), "rlkv_pool_shuffle")


class Cache:
    """Convenience owner: a torch uint8 arena plus the handle, with tensor-checking calls."""

    def __init__(self, n_layers, n_q_heads, n_kv_heads, head_dim, batch, sink, recent, dtype, full_mask,
                 max_len, kernel=RLKV_KERNEL_AUTO, device="cuda:0", arena_fill=None, page_tokens=0, pool_pages=0,
                 prefill_tokens=0, **tuning):
        import torch

        self._torch = torch
        self.device = torch.device(device)
        self.torch_dtype = torch.float32 if dtype == RLKV_F32 else torch.bfloat16
        self.shape = dict(n_layers=n_layers, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, head_dim=head_dim,
                          batch=batch, sink=sink, recent=recent)
        kw = dict(n_layers=n_layers, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, head_dim=head_dim,
                  batch=batch, sink=sink, recent=recent, dtype=dtype, full_mask=full_mask, max_len=max_len,
                  kernel=kernel, device=self.device.index or 0, page_tokens=page_tokens, pool_pages=pool_pages,
                  prefill_tokens=prefill_tokens, **tuning)
        need = rlkv_cache_required_bytes(**kw)
        if need == 0:
            raise RlkvError(RLKV_ERR_INVALID_ARG, "rlkv_cache_required_bytes")
        self.arena = torch.empty(need, dtype=torch.uint8, device=self.device)
        if arena_fill is not None:          # tests: start from a chosen byte pattern
            self.arena.fill_(arena_fill)
            torch.cuda.synchronize(self.device)
        self.handle = rlkv_cache_create(arena_ptr=self.arena.data_ptr(), arena_bytes=need, **kw)

    def close(self):
        if getattr(self, "handle", None):
            rlkv_cache_destroy(self.handle)
            self.handle = None
            self.arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _stream(self) -> int:
        return self._torch.cuda.current_stream(self.device).cuda_stream

    def _ptr(self, t, shape, what):
        if t.device != self.device or t.dtype != self.torch_dtype or not t.is_contiguous():
            raise ValueError(f"{what}: need a contiguous {self.torch_dtype} tensor on {self.device}")
        if tuple(t.shape) != tuple(shape):
            raise ValueError(f"{what}: shape {tuple(t.shape)} != {tuple(shape)}")
        return t.data_ptr()

    def append(self, layer: int, k, v):
        s = self.shape
        n_tokens = k.shape[2]
        shp = (s["batch"], s["n_kv_heads"], n_tokens, s["head_dim"])
        rlkv_append(self.handle, layer, self._ptr(k, shp, "k"), self._ptr(v, shp, "v"), n_tokens, self._stream())

    def append_ragged(self, layer: int, k, v, n_tokens):
        s = self.shape
        stride = k.shape[2]
        shp = (s["batch"], s["n_kv_heads"], stride, s["head_dim"])
        rlkv_append_ragged(self.handle, layer, self._ptr(k, shp, "k"), self._ptr(v, shp, "v"), n_tokens, stride,
                           self._stream())

    def decode_attention(self, layer: int, q, out, softmax_scale: float):
        s = self.shape
        shp = (s["batch"], s["n_q_heads"], s["head_dim"])
        rlkv_decode_attention(self.handle, layer, self._ptr(q, shp, "q"), self._ptr(out, shp, "out"),
                              softmax_scale, self._stream())

    def decode_attention_noalloc(self, layer: int, q, out, softmax_scale: float):
        s = self.shape
        shp = (s["batch"], s["n_q_heads"], s["head_dim"])
        rlkv_decode_attention_noalloc(self.handle, layer, self._ptr(q, shp, "q"), self._ptr(out, shp, "out"),
                                      softmax_scale, self._stream())

    def append_decode(self, layer: int, k, v, q, out, softmax_scale: float):
        s = self.shape
        kshp = (s["batch"], s["n_kv_heads"], 1, s["head_dim"])
        qshp = (s["batch"], s["n_q_heads"], s["head_dim"])
        rlkv_append_decode(self.handle, layer, self._ptr(k, kshp, "k"), self._ptr(v, kshp, "v"),
                           self._ptr(q, qshp, "q"), self._ptr(out, qshp, "out"), softmax_scale, self._stream())

    def append_decode_prepare(self, layer: int):
        rlkv_append_decode_prepare(self.handle, layer, self._stream())

    def append_decode_launch(self, layer: int, k, v, q, out, softmax_scale: float):
        s = self.shape
        kshp = (s["batch"], s["n_kv_heads"], 1, s["head_dim"])
        qshp = (s["batch"], s["n_q_heads"], s["head_dim"])
        rlkv_append_decode_launch(self.handle, layer, self._ptr(k, kshp, "k"), self._ptr(v, kshp, "v"),
                                  self._ptr(q, qshp, "q"), self._ptr(out, qshp, "out"), softmax_scale, self._stream())

    def worklists_built(self) -> int:
        return rlkv_worklists_built(self.handle)

    def prefill_attention(self, layer: int, q, k, v, n_tokens, out, softmax_scale: float):
        s = self.shape
        stride = k.shape[2]
        kshp = (s["batch"], s["n_kv_heads"], stride, s["head_dim"])
        qshp = (s["batch"], s["n_q_heads"], stride, s["head_dim"])
        if len(n_tokens) != s["batch"]:
            raise ValueError("n_tokens must have batch entries")
        rlkv_prefill_attention(self.handle, layer, self._ptr(q, qshp, "q"), self._ptr(k, kshp, "k"),
                               self._ptr(v, kshp, "v"), n_tokens, stride, self._ptr(out, qshp, "out"), softmax_scale,
                               self._stream())

    def set_active(self, active=None):
        if active is not None and len(active) != self.shape["batch"]:
            raise ValueError("active must have batch entries")
        rlkv_set_active(self.handle, active, self._stream())

    def set_gates(self, gates=None):
        if gates is not None and np.asarray(gates).size != self.shape["n_layers"] * self.shape["n_kv_heads"]:
            raise ValueError("gates must have n_layers * n_kv_heads entries")
        rlkv_set_gates(self.handle, gates, self._stream())

    def reset(self, seq: int = -1):
        rlkv_cache_reset(self.handle, seq, self._stream())

    def lengths(self, layer: int) -> np.ndarray:
        return rlkv_get_lengths(self.handle, layer, self.shape["batch"])

    def slot_positions(self, layer: int, kv_head: int, seq: int) -> np.ndarray:
        return rlkv_get_slot_positions(self.handle, layer, kv_head, seq, self.shape["sink"] + self.shape["recent"])

    def profile_enable(self, max_records: int):
        self._prof_max = max_records
        rlkv_profile_enable(self.handle, max_records)

    def profile_collect(self) -> np.ndarray:
        return rlkv_profile_collect(self.handle, self._prof_max)

    def resident_bytes(self) -> int:
        return rlkv_resident_bytes(self.handle)

    def kernel(self) -> int:
        return rlkv_cache_kernel(self.handle)

    def pool_pages_free(self) -> int:
        return rlkv_pool_pages_free(self.handle)

    def pool_shuffle(self, seed: int):
        rlkv_pool_shuffle(self.handle, seed)
