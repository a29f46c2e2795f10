"""Parity at the benchmark's full per-layer sizes, in the launch configuration bench.py times:
caches with the real batch, context lengths, masks and windows of the benchmark workloads
(a few of their layers, since layers are independent and shaped alike), prefilled the way
the benchmark prefills, stepped with the fused append+decode call, and compared with the
CPU oracle on sampled (layer, sequence, KV head) groups - the oracle recomputes those
outputs one by one from the complete seeded history."""
import numpy as np
import pytest
import torch

import bench
import paper_2510_08525_amd as rl
from inputs import workloads

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,layers,steps,fused", [
    ("c2", [0, 5], 3, True),            # Llama shape, B8, ctx 8192, 20 % compressed
    ("c3", [0, 1, 2], 34, True),        # Qwen shape (G = 7), B16, ctx 16384, 60 %; crosses a work-list rebuild
    ("c3", [3], 2, False),              # the two separate calls
    ("c4", [7], 45, True),              # ragged 4k-32k, B32, window 64+512; crosses rebuilds and one ring wrap
    ("c5", [2], 34, True),              # ragged 16k-64k, B64; crosses a rebuild, 13 sequences wrap their ring
])
def test_full_size_sampled_parity(gpu_device, name, layers, steps, fused):
    w = workloads.WORKLOADS[name]
    mask = w.mask()
    cache = bench.build_cache(w, mask, layers, steps)
    bench.fill_cache(cache, w, layers)
    assert cache.kernel() == rl.RLKV_KERNEL_MFMA
    outs = [torch.full((w.batch, w.n_q_heads, w.head_dim), float("nan"), dtype=torch.bfloat16, device="cuda:0")
            for _ in layers]
    for s in range(steps):
        bench.run_step(cache, bench.step_inputs(w, layers, s), outs, w.softmax_scale, fused)
    torch.cuda.synchronize()
    for o in outs:
        assert torch.isfinite(o.float()).all()
    worst, ratio, indices_ok = bench.spot_check(w, mask, layers, cache, outs, steps - 1, n_samples=10, details=True)
    assert indices_ok
    assert ratio <= 1.0, f"{name}: worst abs err {worst:.4g}, {ratio:.2f}x the tolerance"
    # the flat bar of the target, unrelaxed: K, V ~ N(0, 1), so outputs of these workloads stay at unit scale
    assert worst <= 1e-2, f"{name}: worst abs err {worst:.4g} over the flat 1e-2 bar"
    # every sequence advanced by exactly `steps` in every layer
    lengths = np.asarray(w.lengths()) + steps
    for li in range(len(layers)):
        np.testing.assert_array_equal(cache.lengths(li), lengths.astype(np.int32))
    # sequences whose ring index wrapped during these steps (the fused append wrote slot S + R - 1, then slot S):
    # their slot tables against the ring simulation, in every compressed head of the first layer
    import oracle
    r0 = (np.asarray(w.lengths()) - w.sink) % w.recent
    wrapped = [b for b in range(w.batch) if r0[b] + steps >= w.recent]
    if steps >= 34 and name in ("c4", "c5"):
        assert wrapped, "the run was meant to cross a ring wrap"
    for b in wrapped[:4]:
        for h in range(w.n_kv_heads):
            if not mask[layers[0], h]:
                np.testing.assert_array_equal(cache.slot_positions(0, h, b),
                                              oracle.ring_simulate(w.sink, w.recent, int(lengths[b]))[0])
    cache.close()


def test_config1_through_the_benchmark_path(gpu_device):
    """Config 1 (fp32, 1 layer, ctx 1024, 16 + 112) exactly as bench.py would run it: 16 fused steps."""
    w = workloads.WORKLOADS["c1"]
    mask = w.mask()
    cache = bench.build_cache(w, mask, [0], 16)
    bench.fill_cache(cache, w, [0])
    outs = [torch.empty(1, 32, 128, dtype=torch.float32, device="cuda:0")]
    for s in range(16):
        bench.run_step(cache, bench.step_inputs(w, [0], s), outs, w.softmax_scale)
        torch.cuda.synchronize()
        worst, ratio, ok = bench.spot_check(w, mask, [0], cache, outs, s, n_samples=8, details=True)
        assert ok and ratio <= 1.0, f"step {s}: err {worst:.3g}"
    cache.close()


def test_full_size_gated_mixture(gpu_device):
    """Eq. 1 at the benchmark's size: Qwen-shaped layers, every head full with gate 0.35."""
    w = workloads.WORKLOADS["c3"].all_full()
    mask = np.ones((w.n_layers, w.n_kv_heads), dtype=np.uint8)
    layers, steps, gate = [0, 1], 3, 0.35
    cache = bench.build_cache(w, mask, layers, steps)
    bench.fill_cache(cache, w, layers)
    cache.set_gates(np.full(len(layers) * w.n_kv_heads, gate, dtype=np.float32))
    outs = [torch.empty(w.batch, w.n_q_heads, w.head_dim, dtype=torch.bfloat16, device="cuda:0") for _ in layers]
    for s in range(steps):
        bench.run_step(cache, bench.step_inputs(w, layers, s), outs, w.softmax_scale)
    torch.cuda.synchronize()
    worst, ratio, ok = bench.spot_check(w, mask, layers, cache, outs, steps - 1, n_samples=8, details=True, gate=gate)
    assert ok and ratio <= 1.0, f"worst abs err {worst:.4g} ({ratio:.2f}x tolerance)"
    cache.close()


@pytest.mark.parametrize("name,chunk,page", [("c3", 2048, 0), ("c3", 512, 512), ("c4", 1024, 0)])
def test_full_size_chunked_prefill(gpu_device, name, chunk, page):
    """Chunked prefill of a whole benchmark context through rlkv_prefill_attention (one layer, the
    launch configuration bench.py times), sampled rows recomputed by the oracle from the seeded history."""
    w = workloads.WORKLOADS[name]
    res = bench.measure_prefill(w, w.mask(), "cuda:0", chunk, n_layers=1, page_tokens=page, n_samples=6)
    assert res["parity_spot_check_worst_over_tolerance"] <= 1.0, res


def test_full_size_gated_prefill(gpu_device):
    """Eq. 1 at prefill at the benchmark's size: Qwen-shaped layer, every head full with gate 0.35."""
    w = workloads.WORKLOADS["c3"].all_full()
    mask = np.ones((w.n_layers, w.n_kv_heads), dtype=np.uint8)
    res = bench.measure_prefill(w, mask, "cuda:0", 1024, n_layers=1, n_samples=6, gate=0.35)
    assert res["parity_spot_check_worst_over_tolerance"] <= 1.0, res
