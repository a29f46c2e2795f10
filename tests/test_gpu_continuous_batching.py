"""Continuous batching through the C-ABI: slots finish, are reset, re-admitted with a new
prompt (ragged prefill of that slot only) and switched on and off with rlkv_set_active,
while the other slots keep decoding.  Every step is checked against the CPU oracle for the
active slots; inactive slots must keep their output rows, lengths and stores untouched."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_08525_amd as rl
from paper_2510_08525_amd import binding
from harness import to_np, tolerance
from inputs import synth

pytestmark = pytest.mark.gpu

VARIANTS = [(rl.RLKV_F32, rl.RLKV_KERNEL_VALU), (rl.RLKV_BF16, rl.RLKV_KERNEL_VALU), (rl.RLKV_BF16, rl.RLKV_KERNEL_MFMA)]
IDS = ["f32-valu", "bf16-valu", "bf16-mfma"]


@pytest.mark.parametrize("dtype,kernel", VARIANTS, ids=IDS)
def test_slots_join_and_leave(gpu_device, dtype, kernel):
    B, Hq, Hkv, D, S, R, cap = 4, 8, 2, 128, 8, 24, 160
    mask = [1, 0]
    tdt = torch.float32 if dtype == rl.RLKV_F32 else torch.bfloat16
    dev = torch.device("cuda:0")
    scale = 1.0 / np.sqrt(D)
    cache = rl.Cache(1, Hq, Hkv, D, B, S, R, dtype, mask, [cap] * B, kernel=kernel, device=dev)

    rng = np.random.RandomState(7)
    hist = [None] * B          # (k, v) complete history of the slot's current request
    n = np.zeros(B, dtype=np.int64)
    target = np.zeros(B, dtype=np.int64)
    active = np.zeros(B, dtype=np.uint8)
    next_request = 0

    def admit(slot):
        nonlocal next_request
        rid = 1000 * slot + next_request
        next_request += 1
        k = synth.normal(31, synth.T_K, 0, [rid], range(Hkv), 0, cap, D, dtype=tdt, sink_scale=4.0, n_sink_scaled=4)[0]
        v = synth.normal(31, synth.T_V, 0, [rid], range(Hkv), 0, cap, D, dtype=tdt)[0]
        hist[slot] = (k, v)
        prompt = int(rng.randint(1, 70))
        target[slot] = prompt + int(rng.randint(3, 40))
        counts = np.zeros(B, dtype=np.int32)
        counts[slot] = prompt
        kk = torch.zeros(B, Hkv, prompt, D, dtype=tdt)
        vv = torch.zeros_like(kk)
        kk[slot], vv[slot] = k[:, :prompt], v[:, :prompt]
        cache.append_ragged(0, kk.to(dev), vv.to(dev), counts)       # prefill of the newcomer only
        n[slot] = prompt
        active[slot] = 1

    steps_checked = 0
    for step in range(70):
        for slot in range(B):                                         # retire finished requests
            if active[slot] and n[slot] >= target[slot]:
                cache.reset(slot)
                n[slot], active[slot], hist[slot] = 0, 0, None
        for slot in range(B):                                         # admit into free slots, not all at once
            if not active[slot] and rng.rand() < 0.5:
                admit(slot)
        if not active.any():
            cache.set_active(active)
            q = torch.zeros(B, Hq, D, dtype=tdt, device=dev)
            with pytest.raises(rl.RlkvError) as e:                    # nothing to decode
                cache.decode_attention(0, q, torch.zeros_like(q), scale)
            assert e.value.status == binding.RLKV_ERR_STATE
            continue
        cache.set_active(active)
        k_new = torch.zeros(B, Hkv, 1, D, dtype=tdt)
        v_new = torch.zeros_like(k_new)
        for slot in range(B):
            if active[slot]:
                k_new[slot] = hist[slot][0][:, n[slot]:n[slot] + 1]
                v_new[slot] = hist[slot][1][:, n[slot]:n[slot] + 1]
        q = synth.normal(31, synth.T_Q, 0, range(B), range(Hq), step, 1, D, dtype=tdt)[:, :, 0, :].contiguous()
        out = torch.full((B, Hq, D), 7.0, dtype=tdt, device=dev)     # sentinel
        cache.append_decode(0, k_new.to(dev), v_new.to(dev), q.to(dev), out, scale)
        torch.cuda.synchronize()
        n += active
        got = out.float().cpu().numpy().astype(np.float64)
        np.testing.assert_array_equal(cache.lengths(0), n.astype(np.int32))
        for slot in range(B):
            if not active[slot]:
                assert (got[slot] == 7.0).all(), f"step {step}: inactive slot {slot} was written"
                continue
            k, v = hist[slot]
            ref = oracle.decode_attention(to_np(k[None]), to_np(v[None]), [int(n[slot])], mask, to_np(q[slot:slot + 1]),
                                          S, R, scale)[0]
            err = np.abs(got[slot] - ref)
            assert (err <= tolerance(ref, dtype)).all(), f"step {step} slot {slot} n {n[slot]}: err {err.max():.3e}"
            np.testing.assert_array_equal(cache.slot_positions(0, 1, slot), oracle.ring_simulate(S, R, int(n[slot]))[0])
            steps_checked += 1
    assert steps_checked > 100
    cache.set_active(None)          # back to all slots
    cache.close()


def test_set_active_validation(gpu_device):
    cache = rl.Cache(1, 4, 2, 128, 3, 4, 4, rl.RLKV_BF16, [1, 0], [32, 32, 32])
    with pytest.raises(rl.RlkvError) as e:
        cache.set_active([1, 2, 0])
    assert e.value.status == binding.RLKV_ERR_INVALID_ARG
    with pytest.raises(ValueError):
        cache.set_active([1, 0])
    cache.close()
