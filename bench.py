#!/usr/bin/env python3
"""Benchmark of decode attention over a head-mixed KV cache on one MI355X.

One "step" = one pass of the whole hot path over one batch: for every layer, append one
new K/V row per (sequence, KV head) (with ring eviction in compressed heads), then
decode attention for all query heads (work-list build, split-K attention, merge).
One "token" = one sequence advanced by one position through all layers.

    python bench.py [--workload c3] [--steps K] [--warmup W] [--kernel auto|mfma|valu]

prints ONE JSON line: whole-job tokens/s with all inputs resident in HBM, plus
  roofline     - the split-K attention kernel against the 8 TB/s HBM peak: algorithmic bytes
                 per launch / mean launch duration (HIP events around that kernel)
  all_full     - the same shape with every head full (the paper's full-attention baseline)
  cpu_baseline - the CPU oracle timed on this machine's host cores on a bounded sample
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import paper_2510_08525_amd as rl  # noqa: E402
from inputs import synth, workloads  # noqa: E402

HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E, published peak
PREFILL_CHUNK = 512


def log(*a):
    print(*a, file=sys.stderr, flush=True)


# ------------------------------------------------------------------ cache construction

def dtype_code(w) -> int:
    return rl.RLKV_F32 if w.dtype == "f32" else rl.RLKV_BF16


def torch_dtype(w):
    return torch.float32 if w.dtype == "f32" else torch.bfloat16


def build_cache(w, mask: np.ndarray, layers, extra_tokens: int, kernel=rl.RLKV_KERNEL_AUTO, device="cuda:0",
                page_tokens: int = 0):
    """A cache holding `layers` (list of workload layer ids) of workload `w`.  page_tokens > 0:
    full heads paged, the pool sized to the tokens the run caches and handed out in shuffled
    order (the state of a pool after long service)."""
    lengths = w.lengths()
    max_len = [n + extra_tokens for n in lengths]
    sub_mask = np.ascontiguousarray(mask[list(layers)])
    pool = sum(-(-m // page_tokens) for m in max_len) if page_tokens else 0
    cache = rl.Cache(len(layers), w.n_q_heads, w.n_kv_heads, w.head_dim, w.batch, w.sink, w.recent,
                     dtype_code(w), sub_mask, max_len, kernel=kernel, device=device, page_tokens=page_tokens,
                     pool_pages=pool)
    if page_tokens:
        cache.pool_shuffle(w.seed)
    return cache


def gen_rows(w, tensor_id, layer, pos, heads, device):
    """Rows of K / V / Q at per-sequence positions pos [B, n]: [B, heads, n, D]."""
    sink = dict(sink_scale=w.sink_key_scale, n_sink_scaled=w.n_sink_keys) if tensor_id == synth.T_K else {}
    return synth.normal_at(w.seed, tensor_id, layer, range(w.batch), range(heads), pos, w.head_dim,
                           dtype=torch_dtype(w), device=device, **sink)


def fill_cache(cache, w, layers, device="cuda:0", chunk=PREFILL_CHUNK):
    """Prefill every layer with its seeded context through multi-token appends (exercises
    eviction in compressed heads).  Not timed."""
    lengths = np.asarray(w.lengths(), dtype=np.int64)
    max_ctx = int(lengths.max())
    for li, layer in enumerate(layers):
        for p0 in range(0, max_ctx, chunk):
            counts = np.clip(lengths - p0, 0, chunk).astype(np.int32)
            pos = torch.arange(p0, p0 + chunk, device=device)[None, :].expand(w.batch, chunk)
            k = gen_rows(w, synth.T_K, layer, pos, w.n_kv_heads, device)
            v = gen_rows(w, synth.T_V, layer, pos, w.n_kv_heads, device)
            if (counts == chunk).all():
                cache.append(li, k, v)
            else:
                cache.append_ragged(li, k, v, counts)
    torch.cuda.synchronize()


def step_inputs(w, layers, step: int, device="cuda:0"):
    """(k_new, v_new, q) per layer for decode step `step` (position ctx_b + step)."""
    lengths = torch.tensor(w.lengths(), device=device)
    pos = (lengths + step)[:, None]
    out = []
    for layer in layers:
        k = gen_rows(w, synth.T_K, layer, pos, w.n_kv_heads, device)
        v = gen_rows(w, synth.T_V, layer, pos, w.n_kv_heads, device)
        q = gen_rows(w, synth.T_Q, layer, pos, w.n_q_heads, device)[:, :, 0, :].contiguous()
        if w.q_prescaled:
            q = (q.float() / np.sqrt(w.head_dim)).to(q.dtype)
        out.append((k, v, q))
    return out


def run_step(cache, inputs, outs, scale, fused=True):
    for li, (k, v, q) in enumerate(inputs):
        if fused:
            cache.append_decode(li, k, v, q, outs[li], scale)
        else:
            cache.append(li, k, v)
            cache.decode_attention(li, q, outs[li], scale)


def layer_bytes(w, mask_row: np.ndarray, n_after: np.ndarray) -> int:
    """Algorithmic bytes of one decode-attention launch: K/V rows of every head's effective
    history, the query read and the output write."""
    e = 4 if w.dtype == "f32" else 2
    W = w.sink + w.recent
    n_full = int(mask_row.sum())
    n_comp = w.n_kv_heads - n_full
    kv = 2 * w.head_dim * e * (n_full * int(n_after.sum()) + n_comp * int(np.minimum(n_after, W).sum()))
    return kv + 2 * w.batch * w.n_q_heads * w.head_dim * e


def parity_tolerance():
    """The tolerance function of the parity tests (tests/harness.py: the one definition)."""
    tests_dir = os.path.join(ROOT, "tests")
    if tests_dir not in sys.path:
        sys.path.insert(0, tests_dir)
    import harness
    return harness.tolerance


# ------------------------------------------------------------------ timed runs

def time_workload(w, mask, layers, steps, warmup, profile_steps, kernel, device, label, fused=True, gate=None,
                  page_tokens=0):
    """Fills a cache, then: warmup, `steps` timed steps, `profile_steps` steps with per-kernel
    events.  Returns a dict of measurements and the cache + last outputs for spot checks."""
    total_steps = warmup + steps + profile_steps
    t0 = time.time()
    cache = build_cache(w, mask, layers, total_steps, kernel, device, page_tokens)
    fill_cache(cache, w, layers, device)
    if gate is not None:
        cache.set_gates(np.full(len(layers) * w.n_kv_heads, gate, dtype=np.float32))
    log(f"[{label}] cache built and filled in {time.time() - t0:.1f}s "
        f"({cache.resident_bytes() / 2**30:.2f} GiB of K/V stores, {len(layers)} layers)")
    inputs = [step_inputs(w, layers, s, device) for s in range(total_steps)]
    outs = [torch.empty(w.batch, w.n_q_heads, w.head_dim, dtype=torch_dtype(w), device=device) for _ in layers]
    scale = w.softmax_scale
    for s in range(warmup):
        run_step(cache, inputs[s], outs, scale, fused)
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    built0 = cache.worklists_built()
    marks[0].record()
    for i, s in enumerate(range(warmup, warmup + steps)):
        run_step(cache, inputs[s], outs, scale, fused)
        marks[i + 1].record()          # a marker per step (no synchronisation): shows one-off stalls of the machine
    torch.cuda.synchronize()
    ms_total = marks[0].elapsed_time(marks[-1])
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    # work lists planned on the host and copied to the device inside the timed region (a list serves 32 tokens
    # of its layer and the layers take turns, so every step carries its share of that periodic work)
    res = {"ms_per_step": ms_total / steps, "steps": steps, "layers": len(layers),
           "ms_per_step_median": per_step[len(per_step) // 2], "ms_per_step_max": per_step[-1],
           "worklist_rebuilds_timed": cache.worklists_built() - built0}

    # per-kernel durations of the split-K attention kernel (separate steps, not in `value`)
    kernel_ms = None
    if profile_steps > 0:
        cache.profile_enable(profile_steps * len(layers))
        for s in range(warmup + steps, total_steps):
            run_step(cache, inputs[s], outs, scale, fused)
        kernel_ms = cache.profile_collect()
        lengths = np.asarray(w.lengths(), dtype=np.int64)
        nbytes = []
        for s in range(warmup + steps, total_steps):
            for li, layer in enumerate(layers):
                nbytes.append(layer_bytes(w, mask[layer], lengths + s + 1))
        nbytes = np.asarray(nbytes, dtype=np.float64)
        assert len(kernel_ms) == len(nbytes)
        res["kernel_ms_mean"] = float(kernel_ms.mean())
        res["kernel_ms_median"] = float(np.median(kernel_ms))       # (one-off stalls of the machine show in the mean
        res["kernel_ms_max"] = float(kernel_ms.max())               # and the maximum, not in the median)
        if len(kernel_ms) > 2 and kernel_ms.max() > 4.0 * np.median(kernel_ms):
            rest = np.delete(kernel_ms, int(kernel_ms.argmax()))
            res["kernel_ms_note"] = (f"one of the {len(kernel_ms)} timed launches took {kernel_ms.max():.3f} ms (a one-off stall; "
                                     f"it is in ms_per_launch and frac); the others average {rest.mean():.4f} ms = "
                                     f"{float(np.delete(nbytes, int(kernel_ms.argmax())).sum() / (rest.sum() * 1e-3) / 1e9):.0f} GB/s")
        res["kernel_bytes_mean"] = float(nbytes.mean())
        res["kernel_gbps"] = float(nbytes.sum() / (kernel_ms.sum() * 1e-3) / 1e9)
    return res, cache, outs, inputs


def spot_check(w, mask, layers, cache, outs, last_step, n_samples=6, details=False, gate=None):
    """Compares sampled outputs of the last executed step with the CPU oracle (complete
    history regenerated on the CPU from the seeded generator).  Returns the worst absolute
    error; with details=True also the worst error / tolerance ratio (the tolerance of the parity
    tests, tests/harness.py: 1e-5 for fp32; for bf16 1e-2, relaxed to the bf16 half ulp at the
    reference plus an accumulation allowance only from |ref| >= 4 on) and whether the sampled
    lengths and ring slot positions equal the oracle's."""
    import oracle
    tolerance = parity_tolerance()

    rng = np.random.RandomState(1234)
    lengths = np.asarray(w.lengths(), dtype=np.int64)
    worst, worst_ratio, indices_ok = 0.0, 0.0, True
    G = w.group
    for _ in range(n_samples):
        li = int(rng.randint(len(layers)))
        b = int(rng.randint(w.batch))
        h = int(rng.randint(w.n_kv_heads))
        layer = layers[li]
        n = int(lengths[b]) + last_step + 1
        pos = torch.arange(n)[None, :]
        sink = dict(sink_scale=w.sink_key_scale, n_sink_scaled=w.n_sink_keys)
        k = synth.normal_at(w.seed, synth.T_K, layer, [b], [h], pos, w.head_dim, dtype=torch_dtype(w), **sink)
        v = synth.normal_at(w.seed, synth.T_V, layer, [b], [h], pos, w.head_dim, dtype=torch_dtype(w))
        qpos = torch.tensor([[n - 1]])
        q = synth.normal_at(w.seed, synth.T_Q, layer, [b], range(h * G, (h + 1) * G), qpos, w.head_dim,
                            dtype=torch_dtype(w))[:, :, 0, :]
        if w.q_prescaled:
            q = (q.float() / np.sqrt(w.head_dim)).to(q.dtype)
        conv = (lambda t: synth.bf16_bits(t)) if w.dtype == "bf16" else (lambda t: t.numpy())
        if gate is None or not mask[layer, h]:
            ref = oracle.decode_attention(conv(k), conv(v), [n], [int(mask[layer, h])], conv(q.contiguous()),
                                          w.sink, w.recent, w.softmax_scale)
        else:
            ref = oracle.decode_attention_gated(conv(k), conv(v), [n], [gate], conv(q.contiguous()),
                                                w.sink, w.recent, w.softmax_scale)
        got = outs[li][b, h * G:(h + 1) * G].float().cpu().numpy()
        err = np.abs(got - ref[0])
        tol = tolerance(ref[0], dtype_code(w))
        worst = max(worst, float(err.max()))
        worst_ratio = max(worst_ratio, float((err / tol).max()))
        if details:
            indices_ok &= int(cache.lengths(li)[b]) == n
            if not mask[layer, h]:
                indices_ok &= bool((cache.slot_positions(li, h, b) == oracle.ring_simulate(w.sink, w.recent, n)[0]).all())
    return (worst, worst_ratio, indices_ok) if details else worst


# ------------------------------------------------------------------ prefill (reported beside the headline)

MFMA_BF16_PEAK_TFLOPS = 2500.0


def prefill_useful_flops(w, mask_row, n_old, t, gate=None):
    """4 * D flops (score + weighted sum) per admitted (query, key) pair and query head: row i of the
    causal mask admits i + 1 keys, row i of the local mask min(i + 1, S) + min(i + 1 - S, R) (i + 1 if
    i + 1 <= S + R)."""
    i1 = np.arange(n_old, n_old + t, dtype=np.float64) + 1.0          # keys visible to the causal row
    causal = i1.sum()
    local = np.where(i1 <= w.sink + w.recent, i1, w.sink + w.recent).sum()
    n_full = int(mask_row.sum())
    if gate is not None and gate < 1.0:
        causal = causal + local          # a gated full head computes both attentions (Eq. 1)
    return 4.0 * w.head_dim * w.group * (n_full * causal + (len(mask_row) - n_full) * local)


def measure_prefill(w, mask, device, chunk, n_layers=2, kernel=rl.RLKV_KERNEL_AUTO, page_tokens=0, n_samples=1,
                    gate=None):
    """Chunked prefill of the workload's whole context through rlkv_prefill_attention on the first
    n_layers layers: tokens/s of the call (attention + staging + append, scaled to all layers) and
    the attention kernel's useful TFLOP/s against the dense bf16 MFMA peak, from the dispatch's own
    timestamps.  n_samples sampled rows per layer are checked against the oracle (worst absolute
    error, and worst error / tolerance with the tolerance of the parity tests)."""
    import oracle
    tolerance = parity_tolerance()

    if w.dtype != "bf16":
        return None
    layers = list(range(min(n_layers, w.n_layers)))
    lengths = np.asarray(w.lengths(), dtype=np.int64)
    max_len = [int(n) for n in lengths]
    sub_mask = np.ascontiguousarray(mask[layers])
    pool = sum(-(-m // page_tokens) for m in max_len) if page_tokens else 0
    cache = rl.Cache(len(layers), w.n_q_heads, w.n_kv_heads, w.head_dim, w.batch, w.sink, w.recent, dtype_code(w),
                     sub_mask, max_len, kernel=kernel, device=device, page_tokens=page_tokens, pool_pages=pool,
                     prefill_tokens=chunk)
    if gate is not None:
        cache.set_gates(np.full(len(layers) * w.n_kv_heads, gate, dtype=np.float32))
    max_ctx = int(lengths.max())
    n_chunks = -(-max_ctx // chunk)
    cache.profile_enable(n_chunks * len(layers))
    out = torch.empty(w.batch, w.n_q_heads, chunk, w.head_dim, dtype=torch_dtype(w), device=device)
    flops, samples = [], []
    rng = np.random.RandomState(99)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    total_ms = 0.0
    for li, layer in enumerate(layers):
        pick_chunks = [int(rng.randint(n_chunks)) for _ in range(n_samples)]
        for ci, p0 in enumerate(range(0, max_ctx, chunk)):
            counts = np.clip(lengths - p0, 0, chunk).astype(np.int32)
            pos = torch.arange(p0, p0 + chunk, device=device)[None, :].expand(w.batch, chunk)
            k = gen_rows(w, synth.T_K, layer, pos, w.n_kv_heads, device)
            v = gen_rows(w, synth.T_V, layer, pos, w.n_kv_heads, device)
            q = gen_rows(w, synth.T_Q, layer, pos, w.n_q_heads, device)
            if w.q_prescaled:
                q = (q.float() / np.sqrt(w.head_dim)).to(q.dtype)
            ev0.record()
            cache.prefill_attention(li, q, k, v, counts, out, w.softmax_scale)
            ev1.record()
            torch.cuda.synchronize()
            total_ms += ev0.elapsed_time(ev1)
            flops.append(sum(prefill_useful_flops(w, mask[layer], p0, int(c), gate) for c in counts))
            for _ in range(pick_chunks.count(ci)):
                live = [b for b in range(w.batch) if counts[b] > 0]
                b = live[int(rng.randint(len(live)))]
                h = int(rng.randint(w.n_kv_heads))
                c = int(rng.randint(int(counts[b])))
                G = w.group
                samples.append((layer, b, h, p0 + c, out[b, h * G:(h + 1) * G, c].float().cpu().numpy()))
    kernel_ms = cache.profile_collect()
    cache.close()
    flops = np.asarray(flops)
    assert len(kernel_ms) == len(flops)
    worst, worst_ratio = 0.0, 0.0
    conv = synth.bf16_bits
    for layer, b, h, i, got in samples:
        G = w.group
        pos = torch.arange(i + 1)[None, :]
        sink = dict(sink_scale=w.sink_key_scale, n_sink_scaled=w.n_sink_keys)
        k = synth.normal_at(w.seed, synth.T_K, layer, [b], [h], pos, w.head_dim, dtype=torch_dtype(w), **sink)
        v = synth.normal_at(w.seed, synth.T_V, layer, [b], [h], pos, w.head_dim, dtype=torch_dtype(w))
        q = synth.normal_at(w.seed, synth.T_Q, layer, [b], range(h * G, (h + 1) * G), torch.tensor([[i]]), w.head_dim,
                            dtype=torch_dtype(w))
        if w.q_prescaled:
            q = (q.float() / np.sqrt(w.head_dim)).to(q.dtype)
        g_eff = float(mask[layer, h]) if gate is None or not mask[layer, h] else float(gate)
        ref = oracle.prefill_attention(conv(k), conv(v), [i], [1], [g_eff], conv(q.contiguous()),
                                       w.sink, w.recent, w.softmax_scale)[0, :, 0]
        err = np.abs(got - ref)
        worst = max(worst, float(err.max()))
        worst_ratio = max(worst_ratio, float((err / tolerance(ref, dtype_code(w))).max()))
    tokens = float(lengths.sum())
    ms_all_layers = total_ms * (w.n_layers / len(layers))
    tflops = float(flops.sum() / (kernel_ms.sum() * 1e-3) / 1e12)
    # the same per chunk index (summed over the measured layers): later chunks see a longer cached context
    by_chunk = (flops.reshape(len(layers), n_chunks).sum(0) / (kernel_ms.reshape(len(layers), n_chunks).sum(0) * 1e-3)
                / 1e12)
    return {"tokens_per_s": tokens / (ms_all_layers * 1e-3), "chunk": chunk, "layers_measured": len(layers),
            "ms_per_layer": total_ms / len(layers), "parity_spot_check_max_abs_err": worst,
            "parity_spot_check_worst_over_tolerance": worst_ratio,
            "roofline": {"bound": "mfma", "kernel": "prefill_mfma_kernel", "achieved": tflops,
                         "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tflops / MFMA_BF16_PEAK_TFLOPS,
                         "traffic": None, "flops_per_launch": float(flops.mean()),
                         "ms_per_launch": float(kernel_ms.mean()),
                         "tflops_by_chunk": [round(float(x), 1) for x in by_chunk]}}


def cpu_oracle_baseline(w, mask, device="cuda:0", target_seconds=12.0, max_seqs=16):
    """Times the CPU oracle (fp32 variant, as it stands) on a bounded sample of the workload:
    whole layers (all heads) of up to `max_seqs` sequences, one decode step per layer, until
    about `target_seconds` of oracle time.  Returns tokens/s extrapolated to all layers."""
    import oracle

    lengths = np.asarray(w.lengths(), dtype=np.int64)
    n_seq = min(w.batch, max_seqs)
    seqs = list(range(n_seq))
    cap = int(lengths[seqs].max()) + 1
    conv = (lambda t: synth.bf16_bits(t)) if w.dtype == "bf16" else (lambda t: t.numpy())
    sink = dict(sink_scale=w.sink_key_scale, n_sink_scaled=w.n_sink_keys)
    n = (lengths[seqs] + 1).astype(np.int32)
    # decode steps per sampled layer: the query changes, the history does not (the oracle's
    # cost does not depend on the values), so one copy of the history serves several steps
    reps = 16
    elapsed, layers_done = 0.0, 0
    for layer in range(w.n_layers):
        # the complete history of the sampled sequences, from the seeded generator (made on
        # the GPU because it is faster there; the values are the same on either device)
        k = synth.normal(w.seed, synth.T_K, layer, seqs, range(w.n_kv_heads), 0, cap, w.head_dim,
                         dtype=torch_dtype(w), device=device, **sink).cpu()
        v = synth.normal(w.seed, synth.T_V, layer, seqs, range(w.n_kv_heads), 0, cap, w.head_dim,
                         dtype=torch_dtype(w), device=device).cpu()
        kn, vn = conv(k), conv(v)
        for r in range(reps):
            q = synth.normal(w.seed, synth.T_Q, layer, seqs, range(w.n_q_heads), r, 1, w.head_dim,
                             dtype=torch_dtype(w))[:, :, 0, :].contiguous()
            qn = conv(q)
            t0 = time.perf_counter()
            oracle.decode_attention(kn, vn, n, mask[layer], qn, w.sink, w.recent, w.softmax_scale, precision="f32")
            elapsed += time.perf_counter() - t0
        layers_done += 1
        del k, v, kn, vn
        if elapsed >= target_seconds:
            break
    elapsed /= reps
    per_layer = elapsed / layers_done
    tokens_per_s = n_seq / (per_layer * w.n_layers)
    return {"value": tokens_per_s, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{layers_done} layer(s) x {n_seq} sequence(s) of {w.name}, all heads, {reps} decode steps each, "
                      f"fp32 oracle, OpenMP over (sequence, query head); {elapsed * reps:.1f}s of oracle time, "
                      f"extrapolated to {w.n_layers} layers"}


def measured_stream_ceiling(device, gib=4, reps=4):
    """What a plain streaming read reaches on this machine, as a second yardstick beside the nominal
    8 TB/s: the library's probe kernel (128-bit non-temporal loads, no arithmetic) over `gib` GiB,
    best of several grid sizes and `reps` launches each, timed with events on the launching stream."""
    nbytes = gib << 30
    buf = torch.ones(nbytes // 4, dtype=torch.int32, device=device)
    sink = torch.zeros(4, dtype=torch.int32, device=device)
    stream = torch.cuda.current_stream(device).cuda_stream
    n_cu = torch.cuda.get_device_properties(device).multi_processor_count
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    best, best_wg = 0.0, 0
    for per_cu in (1, 2, 4, 8):
        for _ in range(reps):
            ev0.record()
            rl.rlkv_probe_stream_read(buf.data_ptr(), nbytes, sink.data_ptr(), n_cu * per_cu, stream)
            ev1.record()
            torch.cuda.synchronize()
            gbps = nbytes / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
            if gbps > best:
                best, best_wg = gbps, n_cu * per_cu
    del buf, sink
    torch.cuda.empty_cache()
    return {"read_gbps": best, "workgroups": best_wg, "gib": gib}


KERNEL_SOURCES = {"decode_mfma_kernel": ("decode_mfma.hip", "mfma_tile.h", "rlkv_internal.h"),
                  "decode_valu_kernel": ("decode_valu.hip", "rlkv_internal.h")}


def kernel_source_sha16(kernel_name: str) -> str:
    """Fingerprint of the sources a kernel is built from (what a profile summary records beside its figures)."""
    import hashlib

    h = hashlib.sha256()
    for f in KERNEL_SOURCES.get(kernel_name, ()):
        h.update(open(os.path.join(ROOT, "paper_2510_08525_amd", "csrc", f), "rb").read())
    return h.hexdigest()[:16]


def profiled_traffic(kernel_name: str, workload: str):
    """HBM bytes per launch of the dominant kernel as the committed rocprofv3 --pmc summary under profiles/
    states them (FETCH_SIZE + WRITE_SIZE, each scaled by a copy kernel of known size), with the file named as
    the source: the figure is a record of that profiling run, not a measurement of this one.  None when there
    is no summary for the workload, or when the summary was made with other kernel sources than the present
    ones (it records their fingerprint)."""
    import re

    if "@" in workload:
        return None
    rel = os.path.join("profiles", f"{kernel_name}_{workload}_pmc.txt")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None
    text = open(path).read()
    sha = re.search(r"kernel_source_sha16\s*[:=]\s*([0-9a-f]{16})", text)
    if not sha or sha.group(1) != kernel_source_sha16(kernel_name):
        return None
    m = re.search(r"traffic_bytes_per_launch\s*[:=]\s*([0-9.eE+]+)", text)
    return {"bytes": float(m.group(1)), "source": rel + " (rocprofv3 --pmc run of the same kernel sources)"} if m else None


def concurrency_at_budget(w, mask):
    """Pool rebalancing (paper Sec. 4.3, Table 3 "Concur."): how many sequences of the workload's
    mean context fit into the memory the all-full cache needs for its batch, once the masked
    heads only hold sink + recent.  From rlkv_cache_required_bytes; nothing is allocated."""
    ctx = int(np.mean(w.lengths())) + 64

    def need(batch, m):
        return rl.rlkv_cache_required_bytes(n_layers=w.n_layers, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads,
                                            head_dim=w.head_dim, batch=batch, sink=w.sink, recent=w.recent,
                                            dtype=dtype_code(w), full_mask=m, max_len=[ctx] * batch)
    budget = need(w.batch, np.ones_like(mask))
    lo, hi = w.batch, w.batch * 64
    while lo < hi:                      # largest batch whose mixed cache fits the budget
        mid = (lo + hi + 1) // 2
        if need(mid, mask) <= budget:
            lo = mid
        else:
            hi = mid - 1
    return {"budget_gib": budget / 2**30, "context": ctx, "sequences_all_full": w.batch, "sequences_mixed": lo,
            "ratio": lo / w.batch}


_GRAPHS_WARM = False


def measure_graph(w, mask, device, steps, warmup):
    """A decode step recorded once into a HIP graph (rlkv_append_decode_launch of every layer) and replayed, against
    the same step issued call by call (Sec. 4.3: per-layer dispatch overhead).  Both legs run the same work: one
    copy of the step's rows (K, V, Q of all layers, packed) into the fixed buffers a recorded launch reads, then
    the L fused launches; the replayed leg calls rlkv_append_decode_prepare for every layer before each replay.
    The two legs use two caches filled alike.  (fp32 runs on the vector-ALU kernel, whose recorded step is three
    launches per layer: append, attention, merge.)"""
    layers = list(range(w.n_layers))
    L, B, D = w.n_layers, w.batch, w.head_dim
    # the first graph a process replays runs slowly at first (the runtime is still setting up): a throwaway graph
    # is replayed for a quarter of a second before the first measurement, and both legs warm up for at least 40 steps
    global _GRAPHS_WARM
    if not _GRAPHS_WARM:
        x = torch.zeros(1024, device=device)
        g0 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g0):
            for _ in range(8):
                x.add_(1.0)
        t_end = time.perf_counter() + 0.25
        while time.perf_counter() < t_end:
            g0.replay()
        torch.cuda.synchronize()
        del g0, x
        _GRAPHS_WARM = True
    warmup = max(warmup, 40)
    total = warmup + steps
    nk, nq = L * B * w.n_kv_heads * D, L * B * w.n_q_heads * D
    packed = []
    for s in range(total):
        rows = step_inputs(w, layers, s, device)
        packed.append(torch.cat([torch.stack([r[0] for r in rows]).reshape(-1), torch.stack([r[1] for r in rows]).reshape(-1),
                                 torch.stack([r[2] for r in rows]).reshape(-1)]))
    fixed = torch.zeros(2 * nk + nq, dtype=torch_dtype(w), device=device)
    k_s = fixed[:nk].view(L, B, w.n_kv_heads, 1, D)
    v_s = fixed[nk:2 * nk].view(L, B, w.n_kv_heads, 1, D)
    q_s = fixed[2 * nk:].view(L, B, w.n_q_heads, D)
    scale = w.softmax_scale
    results, outs_of = {}, {}
    for leg in ("per_call", "graph"):
        cache = build_cache(w, mask, layers, total, rl.RLKV_KERNEL_AUTO, device)
        fill_cache(cache, w, layers, device)
        outs = torch.zeros(L, B, w.n_q_heads, D, dtype=torch_dtype(w), device=device)
        graph = None
        if leg == "graph":
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for l in range(L):
                    cache.append_decode_launch(l, k_s[l], v_s[l], q_s[l], outs[l], scale)

        def one_step(s):
            fixed.copy_(packed[s])
            if graph is None:
                for l in range(L):
                    cache.append_decode(l, k_s[l], v_s[l], q_s[l], outs[l], scale)
            else:
                for l in range(L):
                    cache.append_decode_prepare(l)
                graph.replay()

        for s in range(warmup):
            one_step(s)
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        ev0.record()
        for s in range(warmup, total):
            one_step(s)
        ev1.record()
        host_ms = (time.perf_counter() - t0) * 1e3 / steps         # host time to issue a step (no waiting)
        torch.cuda.synchronize()
        results[leg] = {"ms_per_step": ev0.elapsed_time(ev1) / steps, "host_issue_ms_per_step": host_ms}
        outs_of[leg] = outs.clone()
        cache.close()
        del cache
        torch.cuda.empty_cache()
    return {"steps": steps, "ms_per_step_per_call": results["per_call"]["ms_per_step"],
            "ms_per_step_graph": results["graph"]["ms_per_step"],
            "host_issue_ms_per_step_per_call": results["per_call"]["host_issue_ms_per_step"],
            "host_issue_ms_per_step_graph": results["graph"]["host_issue_ms_per_step"],
            "outputs_bit_equal": bool(torch.equal(outs_of["per_call"].contiguous().view(torch.uint8),
                                                  outs_of["graph"].contiguous().view(torch.uint8)))}


def measure_equal_memory(w, mask, args, kernel, device, conc, all_full):
    """Pool rebalancing measured (Sec. 4.3, Table 3 "Concur."): the memory the all-full cache needs for the
    workload's batch holds `sequences_mixed` sequences once the masked heads keep only sink + recent; this runs the
    fused decode step at that batch and sets its tokens/s against the all-full run at the original batch."""
    import dataclasses

    wb = dataclasses.replace(w, batch=int(conc["sequences_mixed"]), name=f"{w.name}@B{conc['sequences_mixed']}")
    need = rl.rlkv_cache_required_bytes(n_layers=wb.n_layers, n_q_heads=wb.n_q_heads, n_kv_heads=wb.n_kv_heads,
                                        head_dim=wb.head_dim, batch=wb.batch, sink=wb.sink, recent=wb.recent,
                                        dtype=dtype_code(wb), full_mask=mask,
                                        max_len=[n + args.warmup + args.steps + args.profile_steps for n in wb.lengths()])
    m = measure_workload(wb, args, kernel, device, skip_all_full=True)
    out = {"sequences": wb.batch, "cache_gib": need / 2**30, "budget_gib": conc["budget_gib"],
           "tokens_per_s": m["tokens_per_s"], "ms_per_step": m["ms_per_step"],
           "hbm_frac_whole_step": m["hbm_frac_whole_step"],
           "parity_spot_check_max_abs_err": m["parity_spot_check_max_abs_err"]}
    if "roofline" in m:
        out["kernel_frac"] = m["roofline"]["frac"]
    if all_full is not None:
        out["all_full_sequences"] = w.batch
        out["all_full_tokens_per_s"] = all_full["tokens_per_s"]
        out["speedup_at_equal_memory"] = m["tokens_per_s"] / all_full["tokens_per_s"]
    return out


def resident_layer_subset(w, mask, budget_bytes: float):
    """All layers if they fit the budget, else the longest prefix of layers that does."""
    e = 4 if w.dtype == "f32" else 2
    lengths = np.asarray(w.lengths(), dtype=np.int64) + 64
    W = w.sink + w.recent
    layers, used = [], 0
    for l in range(w.n_layers):
        nf = int(mask[l].sum())
        need = 2 * w.head_dim * e * (nf * int(lengths.sum()) + (w.n_kv_heads - nf) * W * w.batch)
        if used + need > budget_bytes and layers:
            break
        layers.append(l)
        used += need
    return layers


def describe(w, mask) -> str:
    return (f"{w.name}: {w.n_layers} layers x ({w.n_q_heads} q / {w.n_kv_heads} kv heads, head_dim {w.head_dim}), "
            f"batch {w.batch}, context {w.ctx_lo}" + (f"-{w.ctx_hi} ragged" if w.ctx_hi != w.ctx_lo else "")
            + f", {int((mask == 0).sum())}/{mask.size} KV heads compressed (sink {w.sink} + recent {w.recent})")


def measure_workload(w, args, kernel, device, steps=None, all_full=None, skip_all_full=False):
    """Mixed-head run (+ the all-full baseline at the same shape) of one workload.  all_full: an all-full
    measurement of the same shape taken earlier in this run ({"ms_per_step", "tokens_per_s", ...}), reused
    instead of measuring it again."""
    steps = steps or args.steps
    mask = w.mask()
    budget = args.hbm_budget_gib * 2**30
    layers = resident_layer_subset(w, mask, budget)
    scale_layers = w.n_layers / len(layers)
    fused = not args.unfused
    res, cache, outs, inputs = time_workload(w, mask, layers, steps, args.warmup, args.profile_steps,
                                             kernel, device, f"{w.name} mixed", fused, args.gate, args.page_tokens)
    kernel_name = {rl.RLKV_KERNEL_VALU: "decode_valu_kernel", rl.RLKV_KERNEL_MFMA: "decode_mfma_kernel"}[cache.kernel()]
    last_step = args.warmup + steps + args.profile_steps - 1
    max_err = spot_check(w, mask, layers, cache, outs, last_step, gate=args.gate)
    resident_gib = cache.resident_bytes() / 2**30 * scale_layers
    cache.close()
    del cache, outs, inputs
    torch.cuda.empty_cache()

    ms_per_step = res["ms_per_step"] * scale_layers
    lengths = np.asarray(w.lengths(), dtype=np.int64)
    mid = args.warmup + steps // 2
    step_bytes = workloads.algorithmic_bytes_per_step(w, lengths + mid + 1, mask)
    step_gbps = step_bytes / (ms_per_step * 1e-3) / 1e9
    out = {
        "tokens_per_s": w.batch / (ms_per_step * 1e-3), "ms_per_step": ms_per_step, "steps_timed": steps,
        "ms_per_step_median": res["ms_per_step_median"] * scale_layers, "ms_per_step_max": res["ms_per_step_max"] * scale_layers,
        "config": {"workload": describe(w, mask), "compressed_fraction": float((mask == 0).mean()),
                   "kernel": kernel_name, "layers_resident": len(layers), "kv_resident_gib": resident_gib,
                   "gate_on_full_heads": args.gate, "page_tokens": args.page_tokens or None},
        "hbm_gbps_whole_step": step_gbps, "hbm_frac_whole_step": step_gbps / HBM_PEAK_GBPS,
        "worklist_rebuilds_timed": res["worklist_rebuilds_timed"],
        "parity_spot_check_max_abs_err": max_err,
    }
    if "kernel_gbps" in res:
        out["roofline"] = {"bound": "hbm", "kernel": kernel_name, "achieved": res["kernel_gbps"],
                           "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": res["kernel_gbps"] / HBM_PEAK_GBPS,
                           "traffic": None,
                           "bytes_per_launch": res["kernel_bytes_mean"], "ms_per_launch": res["kernel_ms_mean"],
                           "ms_per_launch_median": res["kernel_ms_median"], "ms_per_launch_max": res["kernel_ms_max"]}
        if "kernel_ms_note" in res:
            out["roofline"]["note"] = res["kernel_ms_note"]
        traffic = profiled_traffic(kernel_name, w.name)
        if traffic is not None:
            # not measured by this run: counters need rocprofv3 around the process
            out["roofline"]["traffic"] = traffic["bytes"]
            out["roofline"]["traffic_source"] = traffic["source"]
    lengths_mid = lengths + mid + 1
    if all_full is not None:
        bytes_f = workloads.algorithmic_bytes_per_step(w.all_full(), lengths_mid, np.ones_like(mask))
        out["all_full"] = dict(all_full, shared_with="the all-full run of the same shape earlier in this line")
        out["speedup_vs_all_full"] = all_full["ms_per_step"] / ms_per_step
        out["closed_form_speedup"] = bytes_f / step_bytes
    elif not args.skip_all_full and not skip_all_full:
        wf = w.all_full()
        mask_f = np.ones_like(mask)
        layers_f = resident_layer_subset(wf, mask_f, budget)
        res_f, cache_f, outs_f, inputs_f = time_workload(wf, mask_f, layers_f, steps, args.warmup,
                                                         args.profile_steps, kernel, device, f"{w.name} all-full", fused,
                                                         page_tokens=args.page_tokens)
        cache_f.close()
        del cache_f, outs_f, inputs_f
        torch.cuda.empty_cache()
        ms_f = res_f["ms_per_step"] * (w.n_layers / len(layers_f))
        bytes_f = workloads.algorithmic_bytes_per_step(wf, lengths + mid + 1, mask_f)
        out["all_full"] = {"tokens_per_s": w.batch / (ms_f * 1e-3), "ms_per_step": ms_f,
                           "layers_resident": len(layers_f),
                           "scaled_from_resident_layers": len(layers_f) != w.n_layers,
                           "hbm_gbps_whole_step": bytes_f / (ms_f * 1e-3) / 1e9,
                           "kernel_gbps": res_f.get("kernel_gbps")}
        out["speedup_vs_all_full"] = ms_f / ms_per_step
        out["closed_form_speedup"] = bytes_f / step_bytes
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3", choices=sorted(workloads.WORKLOADS))
    ap.add_argument("--pct", type=int, default=None, help="override the compressed-head percentage")
    ap.add_argument("--also", default="c2,c4@0,c4@20,c4@40,c4,c5",
                    help="comma-separated further workloads measured (shorter) and reported under \"also\"; "
                         "name@pct = that workload with pct %% of the KV heads compressed; \"none\" for none")
    ap.add_argument("--graph-workloads", default="c1,c2,c3",
                    help="workloads whose decode step is also timed as a recorded HIP graph against the per-call "
                         "path, reported under \"graph\"; \"none\" for none")
    ap.add_argument("--skip-graph", action="store_true")
    ap.add_argument("--skip-equal-memory", action="store_true")
    ap.add_argument("--gate", type=float, default=None,
                    help="Eq. 1 gate in [0, 1] set on every full head (mixed attention of the head-identification "
                         "phase); default: binary heads")
    ap.add_argument("--page-tokens", type=int, default=0,
                    help="page the full heads (Sec. 4.3) with pages of this many tokens from a shuffled pool; "
                         "default 0: contiguous per-sequence stores")
    ap.add_argument("--prefill-chunk", type=int, default=2048,
                    help="also measure chunked prefill attention of the workload's context (two layers) with "
                         "chunks of this many tokens, reported under \"prefill\"; 0 to skip")
    ap.add_argument("--prefill-also", default="c4",
                    help="further workloads whose chunked prefill is measured beside the headline one's (comma list, none)")
    ap.add_argument("--prefill-single-ctx", type=int, default=131072,
                    help="also prefill one sequence of this many tokens alone (one layer), reported under "
                         "\"prefill\".\"single_sequence\"; 0 to skip")
    ap.add_argument("--kernel", default="auto", choices=["auto", "valu", "mfma"])
    ap.add_argument("--profile-steps", type=int, default=2)
    ap.add_argument("--skip-all-full", action="store_true")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--unfused", action="store_true", help="separate rlkv_append + rlkv_decode_attention calls")
    ap.add_argument("--hbm-budget-gib", type=float, default=200.0)
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain elementwise copy of 1 GiB (reads 1 GiB, writes 1 GiB) three times, so "
                         "that a rocprofv3 --pmc run of this command holds a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU (the HIP library has no CPU fallback)")
    rl.load_library()
    device = "cuda:0"
    torch.cuda.set_device(0)
    if args.calibration_copy:
        src = torch.ones(1 << 28, dtype=torch.int32, device=device)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1, out=dst)      # vectorized elementwise kernel: 2^30 bytes in, 2^30 bytes out
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    kernel = {"auto": rl.RLKV_KERNEL_AUTO, "valu": rl.RLKV_KERNEL_VALU, "mfma": rl.RLKV_KERNEL_MFMA}[args.kernel]
    w = workloads.WORKLOADS[args.workload]
    if args.pct is not None:
        w = w.with_pct(args.pct)
    m = measure_workload(w, args, kernel, device)
    m_headline = m
    line = {
        "metric": "decode_attention_tokens_per_s", "value": m["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": m["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
    }
    line.update({k: v for k, v in m.items() if k not in ("tokens_per_s", "ms_per_step")})
    mask = w.mask()

    # the same measurement on further workloads (shorter), reported beside the headline one.  "c4@20" = workload c4
    # with 20 % of the KV heads compressed; entries of one shape share one all-full run ("@0" is that run).
    also, full_runs = {}, {}
    for entry in [n for n in args.also.split(",") if n and n != "none" and n != args.workload]:
        name, _, pct = entry.partition("@")
        wa = workloads.WORKLOADS[name]
        if pct:
            wa = wa.with_pct(int(pct))
        elif args.pct is not None:
            wa = wa.with_pct(args.pct)
        steps_a = max(4, args.steps // 2)
        if pct and int(pct) == 0:
            r = measure_workload(wa, args, kernel, device, steps=steps_a, skip_all_full=True)
            r["speedup_vs_all_full"], r["closed_form_speedup"] = 1.0, 1.0
            full_runs[name] = {"tokens_per_s": r["tokens_per_s"], "ms_per_step": r["ms_per_step"],
                               "layers_resident": r["config"]["layers_resident"],
                               "scaled_from_resident_layers": r["config"]["layers_resident"] != wa.n_layers,
                               "hbm_gbps_whole_step": r["hbm_gbps_whole_step"],
                               "kernel_gbps": r.get("roofline", {}).get("achieved")}
        else:
            r = measure_workload(wa, args, kernel, device, steps=steps_a, all_full=full_runs.get(name))
            if "all_full" in r and name not in full_runs:
                full_runs[name] = {k: v for k, v in r["all_full"].items() if k != "shared_with"}
        also[entry] = r
    if also:
        line["also"] = also

    if args.prefill_chunk > 0:
        pre = measure_prefill(w, mask, device, args.prefill_chunk, kernel=kernel, page_tokens=args.page_tokens,
                              gate=args.gate)
        if pre is not None:
            line["prefill"] = pre
            if args.prefill_single_ctx > 0 and args.gate is None:
                # one long prompt alone: too few long workgroups for the chip unless the library divides them
                import dataclasses
                w1 = dataclasses.replace(w, batch=1, ctx_lo=args.prefill_single_ctx, ctx_hi=args.prefill_single_ctx)
                one = measure_prefill(w1, mask, device, args.prefill_chunk, n_layers=1, kernel=kernel,
                                      page_tokens=args.page_tokens)
                r1 = one["roofline"]
                pre["single_sequence"] = {"context": args.prefill_single_ctx, "tokens_per_s": one["tokens_per_s"],
                                          "ms_per_layer": one["ms_per_layer"], "tflops": r1["achieved"],
                                          "tflops_last_chunk": r1["tflops_by_chunk"][-1],
                                          "parity_spot_check_worst_over_tolerance":
                                              one["parity_spot_check_worst_over_tolerance"]}
            # the same on further workloads (their own masks; two layers each)
            for name in [n for n in args.prefill_also.split(",") if n and n != "none" and n != args.workload]:
                if args.gate is not None or args.page_tokens:
                    break
                torch.cuda.empty_cache()
                wp = workloads.WORKLOADS[name]
                other = measure_prefill(wp, wp.mask(), device, args.prefill_chunk, kernel=kernel)
                if other is not None:
                    pre.setdefault("also", {})[name] = {
                        "workload": describe(wp, wp.mask()), "tokens_per_s": other["tokens_per_s"],
                        "ms_per_layer": other["ms_per_layer"], "roofline": other["roofline"],
                        "parity_spot_check_worst_over_tolerance": other["parity_spot_check_worst_over_tolerance"]}
        torch.cuda.empty_cache()

    conc = concurrency_at_budget(w, mask)
    line["concurrency_at_equal_memory"] = conc
    if not args.skip_equal_memory and args.gate is None and "all_full" in m_headline:
        line["equal_memory"] = measure_equal_memory(w, mask, args, kernel, device, conc, m_headline["all_full"])
    if not args.skip_graph and args.gate is None and not args.page_tokens:
        graphs = {}
        for name in [n for n in args.graph_workloads.split(",") if n and n != "none"]:
            wg = workloads.WORKLOADS[name]
            g = measure_graph(wg, wg.mask(), device, args.steps, args.warmup)
            graphs[name] = g
        line["graph"] = graphs
    ceiling = measured_stream_ceiling(device)
    line["measured_stream_ceiling"] = ceiling
    if "roofline" in line:
        line["roofline"]["frac_of_measured_ceiling"] = line["roofline"]["achieved"] / ceiling["read_gbps"]
    for m in line.get("also", {}).values():
        if "roofline" in m:
            m["roofline"]["frac_of_measured_ceiling"] = m["roofline"]["achieved"] / ceiling["read_gbps"]
    if not args.skip_cpu:
        line["cpu_baseline"] = cpu_oracle_baseline(w, mask, device)

    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
