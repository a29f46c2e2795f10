"""Randomised schedules through the C-ABI: random shapes, windows and a random sequence of
uniform / ragged appends, fused steps, resets with refill, active-set changes and gate
changes; after every attention call the outputs, lengths and ring slots are compared with
the oracle.  Seeds are fixed, so a failure names its seed and step."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_08525_amd as rl
from harness import to_np, tolerance
from inputs import synth

pytestmark = pytest.mark.gpu

SHAPES = [(32, 8), (28, 4), (8, 8), (7, 1), (16, 1), (12, 4), (10, 2)]
VARIANTS = [(rl.RLKV_F32, rl.RLKV_KERNEL_VALU), (rl.RLKV_BF16, rl.RLKV_KERNEL_VALU), (rl.RLKV_BF16, rl.RLKV_KERNEL_MFMA)]


@pytest.mark.parametrize("seed", list(range(12)))
def test_random_schedule(gpu_device, seed):
    run_schedule(seed, paged=False)


@pytest.mark.parametrize("seed", list(range(100, 108)))
def test_random_schedule_paged(gpu_device, seed):
    """Same schedules over paged full heads (Sec. 4.3): small pages from a shuffled pool, so that
    sequences cross page boundaries all the time and resets hand pages from one slot to another;
    also checks the free-page count against the lengths."""
    run_schedule(seed, paged=True)


def run_schedule(seed, paged):
    rng = np.random.RandomState(1000 + seed)
    dtype, kernel = VARIANTS[2 if paged else seed % 3]
    Hq, Hkv = SHAPES[rng.randint(len(SHAPES))]
    B = int(rng.randint(1, 5))
    S = int(rng.choice([0, 1, 4, 16, 33]))
    R = int(rng.choice([1, 3, 17, 32, 70]))
    cap = int(rng.randint(150, 700))
    D = 128
    mask = rng.randint(0, 2, size=Hkv).astype(np.uint8)
    tdt = torch.float32 if dtype == rl.RLKV_F32 else torch.bfloat16
    dev = torch.device("cuda:0")
    scale = float(rng.choice([1.0 / np.sqrt(D), 0.05, 0.2]))
    page = int(rng.choice([32, 64, 128])) if paged else 0
    pool = B * (-(-cap // page)) if paged else 0
    can_prefill = kernel == rl.RLKV_KERNEL_MFMA
    cache = rl.Cache(1, Hq, Hkv, D, B, S, R, dtype, mask, [cap] * B, kernel=kernel, device=dev, page_tokens=page,
                     pool_pages=pool, prefill_tokens=96 if can_prefill else 0)
    if paged:
        cache.pool_shuffle(seed)
    gen = [0] * B                                     # request generation per slot (new history after a reset)

    def history(b):
        rid = b * 100 + gen[b]
        k = synth.normal(seed, synth.T_K, 0, [rid], range(Hkv), 0, cap, D, dtype=tdt, sink_scale=4.0, n_sink_scaled=4)[0]
        v = synth.normal(seed, synth.T_V, 0, [rid], range(Hkv), 0, cap, D, dtype=tdt)[0]
        return k, v

    hist = [history(b) for b in range(B)]
    n = np.zeros(B, dtype=np.int64)
    active = np.ones(B, dtype=np.uint8)
    gates = np.ones(Hkv, dtype=np.float32)

    def rows(counts):
        stride = int(max(1, counts.max()))
        k = torch.zeros(B, Hkv, stride, D, dtype=tdt)
        v = torch.zeros_like(k)
        for b in range(B):
            c = int(min(counts[b], cap - n[b]))        # a slot at capacity can only be a skipped (inactive) one
            k[b, :, :c] = hist[b][0][:, n[b]:n[b] + c]
            v[b, :, :c] = hist[b][1][:, n[b]:n[b] + c]
        return k.to(dev), v.to(dev)

    def check(out, q, step):
        got = out.float().cpu().numpy().astype(np.float64)
        np.testing.assert_array_equal(cache.lengths(0), n.astype(np.int32), err_msg=f"seed {seed} step {step}")
        if paged:
            assert cache.pool_pages_free() == pool - int(sum(-(-int(x) // page) for x in n)), f"seed {seed} step {step}"
        eff = [float(g) if m else 0.0 for g, m in zip(gates, mask)]
        for b in range(B):
            if not active[b]:
                assert (got[b] == 3.0).all(), f"seed {seed} step {step}: inactive slot {b} written"
                continue
            ref = oracle.decode_attention_gated(to_np(hist[b][0][None]), to_np(hist[b][1][None]), [int(n[b])], eff,
                                                to_np(q[b:b + 1]), S, R, scale)[0]
            err = np.abs(got[b] - ref)
            assert (err <= tolerance(ref, dtype)).all(), \
                f"seed {seed} step {step} slot {b} n {n[b]} (Hq {Hq} Hkv {Hkv} S {S} R {R} mask {mask}): {err.max():.3e}"
            for h in range(Hkv):
                if not mask[h]:
                    np.testing.assert_array_equal(cache.slot_positions(0, h, b), oracle.ring_simulate(S, R, int(n[b]))[0])

    checks = 0
    for step in range(45):
        op = rng.choice(["fused", "fused", "fused", "uniform", "ragged", "decode", "reset", "active", "gates", "prefill"])
        room = cap - n
        if op == "uniform":
            t = int(rng.randint(1, 40))
            if (room[active == 1] < t).any() or not active.any():
                continue
            counts = np.where(active == 1, t, 0)
            k, v = rows(np.full(B, t))                 # rows for inactive slots are ignored
            for b in range(B):
                if not active[b]:
                    k[b] = 0
            cache.append(0, k, v)
            n += counts
        elif op == "ragged":
            counts = np.minimum(rng.randint(0, 2 * (S + R) + 5, size=B), room).astype(np.int64)
            if counts.max() == 0:
                continue
            k, v = rows(counts)
            cache.append_ragged(0, k, v, counts.astype(np.int32))
            n += counts
        elif op == "prefill":
            if not can_prefill:
                continue
            counts = np.minimum(rng.randint(0, 97, size=B), room).astype(np.int64)
            if counts.max() == 0:
                continue
            stride = int(counts.max())
            k, v = rows(counts)
            qp = synth.normal(seed, synth.T_Q, 0, range(B), range(Hq), 5000 * (step + 1), stride, D, dtype=tdt).contiguous()
            outp = torch.full((B, Hq, stride, D), 3.0, dtype=tdt, device=dev)
            cache.prefill_attention(0, qp.to(dev), k, v, counts.astype(np.int32), outp, scale)
            torch.cuda.synchronize()
            eff = [float(g) if m else 0.0 for g, m in zip(gates, mask)]
            got = outp.float().cpu().numpy().astype(np.float64)
            for b in range(B):
                c = int(counts[b])
                assert (got[b, :, c:] == 3.0).all(), f"seed {seed} step {step}: rows past the chunk of slot {b} written"
                if c == 0:
                    continue
                ref = oracle.prefill_attention(to_np(hist[b][0][None]), to_np(hist[b][1][None]), [int(n[b])], [c], eff,
                                               to_np(qp[b:b + 1, :, :c].contiguous()), S, R, scale)[0]
                err = np.abs(got[b, :, :c] - ref)
                assert (err <= tolerance(ref, dtype)).all(), \
                    f"seed {seed} step {step} prefill slot {b} n {n[b]} + {c} (S {S} R {R} mask {mask} gates {gates}): {err.max():.3e}"
            n += counts
            checks += 1
        elif op == "reset":
            b = int(rng.randint(B))
            cache.reset(b)
            n[b] = 0
            gen[b] += 1
            hist[b] = history(b)
            c = np.zeros(B, dtype=np.int64)
            c[b] = int(rng.randint(1, min(cap, 3 * (S + R) + 10)))
            k, v = rows(c)
            cache.append_ragged(0, k, v, c.astype(np.int32))   # refill the slot with its new request
            n += c
        elif op == "active":
            active = rng.randint(0, 2, size=B).astype(np.uint8)
            if not active.any():
                active[int(rng.randint(B))] = 1
            cache.set_active(active)
        elif op == "gates":
            gates = rng.choice([0.0, 0.25, 0.6, 1.0], size=Hkv).astype(np.float32)
            cache.set_gates(gates)
        elif op in ("fused", "decode"):
            if (n[active == 1] < 1).any() and op == "decode":
                continue
            if op == "fused" and (room[active == 1] < 1).any():
                continue
            q = synth.normal(seed, synth.T_Q, 0, range(B), range(Hq), step, 1, D, dtype=tdt)[:, :, 0, :].contiguous()
            out = torch.full((B, Hq, D), 3.0, dtype=tdt, device=dev)
            if op == "fused":
                k, v = rows(np.ones(B, dtype=np.int64))
                cache.append_decode(0, k, v, q.to(dev), out, scale)
                n += active
            else:
                cache.decode_attention(0, q.to(dev), out, scale)
            torch.cuda.synchronize()
            check(out, q, step)
            checks += 1
    assert checks >= 5, f"seed {seed}: only {checks} attention calls"
    cache.close()
