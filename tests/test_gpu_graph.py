"""A recorded decode step: rlkv_append_decode_launch of every layer captured into a HIP graph once and replayed,
with rlkv_append_decode_prepare before each replay (Sec. 4.3: the per-layer dispatch overhead is what separates
the measured from the theoretical speedup).  Every replay is compared bit for bit with the per-call path
(rlkv_append_decode on a second cache fed the same rows) and with the oracle; eager work and synchronisations
sit between the replays, and the run is long enough to cross several work-list rebuilds and ring wraps."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_08525_amd as rl
from paper_2510_08525_amd import binding
from harness import to_np, tolerance
from inputs import synth

pytestmark = pytest.mark.gpu

BF16, F32, MFMA, VALU = rl.RLKV_BF16, rl.RLKV_F32, rl.RLKV_KERNEL_MFMA, rl.RLKV_KERNEL_VALU


def _setup(L, Hq, Hkv, B, S, R, mask, ctx, steps, seed, page_tokens=0, dtype=BF16, kernel=MFMA):
    dev = torch.device("cuda:0")
    D = 128
    cap = max(ctx) + steps
    tdt = torch.bfloat16 if dtype == BF16 else torch.float32
    hist = []
    for l in range(L):
        k = synth.normal(seed, synth.T_K, l, range(B), range(Hkv), 0, cap, D, dtype=tdt, sink_scale=4.0,
                         n_sink_scaled=4)
        v = synth.normal(seed, synth.T_V, l, range(B), range(Hkv), 0, cap, D, dtype=tdt)
        hist.append((k, v))
    caches = []
    for _ in range(2):
        pool = sum(-(-(c + steps) // page_tokens) for c in ctx) if page_tokens else 0
        c = rl.Cache(L, Hq, Hkv, D, B, S, R, dtype, mask, [cap] * B, kernel=kernel, device=dev, page_tokens=page_tokens,
                     pool_pages=pool)
        for l in range(L):
            k0 = torch.zeros(B, Hkv, max(ctx), D, dtype=tdt)
            v0 = torch.zeros_like(k0)
            for b in range(B):
                k0[b, :, :ctx[b]] = hist[l][0][b, :, :ctx[b]]
                v0[b, :, :ctx[b]] = hist[l][1][b, :, :ctx[b]]
            c.append_ragged(l, k0.to(dev), v0.to(dev), ctx)
        caches.append(c)
    return dev, D, hist, caches


@pytest.mark.parametrize("page_tokens,dtype,kernel", [(0, BF16, MFMA), (64, BF16, MFMA), (0, F32, VALU), (0, BF16, VALU)],
                         ids=["contiguous", "paged", "f32 vector-ALU kernel", "bf16 vector-ALU kernel"])
def test_replayed_step_matches_per_call_path_and_oracle(gpu_device, page_tokens, dtype, kernel):
    """(With the vector-ALU kernel a recorded step is three launches - append, attention, merge - and the
    per-call leg takes the two separate calls rlkv_append and rlkv_decode_attention.)"""
    L, Hq, Hkv, B, S, R = 3, 28, 4, 4, 8, 24
    mask = np.array([[1, 0, 0, 1], [0, 0, 1, 0], [1, 1, 0, 0]], dtype=np.uint8)
    ctx, steps, seed = [1500, 77, 2300, 640], 70, 501
    dev, D, hist, (per_call, replayed) = _setup(L, Hq, Hkv, B, S, R, mask, ctx, steps, seed, page_tokens, dtype, kernel)
    scale = 1.0 / np.sqrt(D)
    tdt = torch.bfloat16 if dtype == BF16 else torch.float32
    bits = torch.int16 if dtype == BF16 else torch.int32
    k_s = [torch.zeros(B, Hkv, 1, D, dtype=tdt, device=dev) for _ in range(L)]
    v_s = [torch.zeros_like(k_s[0]) for _ in range(L)]
    q_s = [torch.zeros(B, Hq, D, dtype=tdt, device=dev) for _ in range(L)]
    out_s = [torch.zeros(B, Hq, D, dtype=tdt, device=dev) for _ in range(L)]
    out_ref = [torch.zeros(B, Hq, D, dtype=tdt, device=dev) for _ in range(L)]

    # the host half may not be recorded; a launch that runs at once needs a prepared step
    with pytest.raises(rl.RlkvError) as e:
        replayed.append_decode_launch(0, k_s[0], v_s[0], q_s[0], out_s[0], scale)
    assert e.value.status == binding.RLKV_ERR_STATE

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        with pytest.raises(rl.RlkvError) as e:
            replayed.append_decode_prepare(0)
        assert e.value.status == binding.RLKV_ERR_STATE
        for l in range(L):
            replayed.append_decode_launch(l, k_s[l], v_s[l], q_s[l], out_s[l], scale)
    torch.cuda.synchronize()
    assert replayed.lengths(0).tolist() == ctx          # recording ran nothing

    n = np.asarray(ctx, dtype=np.int64)
    built_before = replayed.worklists_built()
    for s in range(steps):
        qs = []
        for l in range(L):
            k, v = hist[l]
            kn = torch.stack([k[b, :, n[b]:n[b] + 1] for b in range(B)]).contiguous()
            vn = torch.stack([v[b, :, n[b]:n[b] + 1] for b in range(B)]).contiguous()
            q = synth.normal(seed, synth.T_Q, l, range(B), range(Hq), s, 1, D, dtype=tdt)[:, :, 0, :].contiguous()
            qs.append(q)
            k_s[l].copy_(kn)
            v_s[l].copy_(vn)
            q_s[l].copy_(q)
            if kernel == MFMA:
                per_call.append_decode(l, k_s[l], v_s[l], q_s[l], out_ref[l], scale)
            else:
                per_call.append(l, k_s[l], v_s[l])
                per_call.decode_attention(l, q_s[l], out_ref[l], scale)
        for l in range(L):
            replayed.append_decode_prepare(l)
        graph.replay()
        torch.cuda.synchronize()                        # and eager work (the copies above) between replays
        n = n + 1
        for l in range(L):
            assert torch.equal(out_s[l].view(bits), out_ref[l].view(bits)), f"step {s} layer {l}"
        if s % 9 == 0 or s == steps - 1:
            for l in range(L):
                ref = oracle.decode_attention(to_np(hist[l][0]), to_np(hist[l][1]), n, mask[l], to_np(qs[l]), S, R, scale)
                err = np.abs(out_s[l].float().cpu().numpy() - ref)
                assert (err <= tolerance(ref, dtype)).all(), f"step {s} layer {l}: max err {err.max():.3e}"
    # lengths and ring slots after 70 replays (R = 24: every ring has wrapped twice more)
    for l in range(L):
        np.testing.assert_array_equal(replayed.lengths(l), n.astype(np.int32))
        for h in range(Hkv):
            if mask[l, h]:
                continue
            for b in range(B):
                np.testing.assert_array_equal(replayed.slot_positions(l, h, b), oracle.ring_simulate(S, R, int(n[b]))[0])
    # the lists were refreshed on the way (a list serves 32 tokens), by the prepare calls, outside the graph
    assert replayed.worklists_built() - built_before >= 2 * L
    if page_tokens:
        assert replayed.pool_pages_free() == per_call.pool_pages_free()
    per_call.close()
    replayed.close()


def test_rebuilds_are_spread_over_the_steps(gpu_device):
    """A list serves 32 tokens; the layers take turns, so no step plans all of them at once (after the first)."""
    L, Hq, Hkv, B = 8, 4, 2, 2
    mask = np.tile(np.array([1, 0], dtype=np.uint8), (L, 1))
    dev = torch.device("cuda:0")
    c = rl.Cache(L, Hq, Hkv, 128, B, 4, 28, BF16, mask, [200] * B)
    k = torch.randn(B, Hkv, 40, 128, device=dev).to(torch.bfloat16)
    for l in range(L):
        c.append(l, k, k)
    k1 = k[:, :, :1].contiguous()
    q = torch.randn(B, Hq, 128, device=dev).to(torch.bfloat16)
    out = torch.empty_like(q)
    per_step = []
    for s in range(100):
        before = c.worklists_built()
        for l in range(L):
            c.append_decode(l, k1, k1, q, out, 0.1)
        per_step.append(c.worklists_built() - before)
    torch.cuda.synchronize()
    assert per_step[0] == L                      # nothing was planned before the first step
    assert max(per_step[1:]) <= 1                # 8 layers over 32 steps: at most one a step
    assert sum(per_step[33:97]) == 2 * L         # and each layer once per 32 steps
    assert c.lengths(L - 1).tolist() == [140, 140]
    c.close()
