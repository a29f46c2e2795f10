"""GPU parity: the HIP path (through the C-ABI) against the CPU oracle, element by element
on the same seeded inputs.  Ring slot indices and lengths bit-exact; outputs within the
tolerances written in tests/harness.py."""
import numpy as np
import pytest
import torch

import paper_2510_08525_amd as rl
from paper_2510_08525_amd import binding
from harness import Case

pytestmark = pytest.mark.gpu

VALU, MFMA = rl.RLKV_KERNEL_VALU, rl.RLKV_KERNEL_MFMA
BF16, F32 = rl.RLKV_BF16, rl.RLKV_F32
VARIANTS = [(F32, VALU), (BF16, VALU), (BF16, MFMA)]
IDS = ["f32-valu", "bf16-valu", "bf16-mfma"]


def test_library_is_loaded_in_process(gpu_device):
    rl.load_library()
    assert any("librlkv.so" in l for l in open("/proc/self/maps"))


def test_config1_fp32_16_steps(gpu_device):
    """32 q / 8 kv heads, fp32, ctx 1024, heads 0-3 full / 4-7 compressed (16 + 112),
    Q pre-scaled by 1/sqrt(128), 16 decode steps appending one K/V each."""
    c = Case(Hq=32, Hkv=8, B=1, S=16, R=112, dtype=F32, kernel=VALU, mask=[1, 1, 1, 1, 0, 0, 0, 0],
             cap=1024 + 16, seed=251008526, scale=1.0, q_prescale=1.0 / np.sqrt(128.0), sink_keys=False)
    c.append([512])
    c.append([512])
    c.check_indices()
    worst = 0.0
    for step in range(16):
        c.append([1])
        c.check_indices()
        worst = max(worst, c.check_decode(step, f"c1 step {step}"))
    assert c.n[0] == 1040
    print("config 1 worst abs err", worst)
    c.close()


@pytest.mark.parametrize("dtype,kernel", VARIANTS, ids=IDS)
@pytest.mark.parametrize("Hq,Hkv", [(32, 8), (28, 4), (8, 8), (7, 1), (16, 1)])
def test_token_by_token_through_sink_window_and_wraps(gpu_device, dtype, kernel, Hq, Hkv):
    """Lengths 1..40 with S=4, R=8: crosses n<S, n==S, n==S+R, S+R+1 and wraps the ring 4x."""
    mask = [(h % 2) for h in range(Hkv)]
    c = Case(Hq=Hq, Hkv=Hkv, B=2, S=4, R=8, dtype=dtype, kernel=kernel, mask=mask, cap=64, seed=3)
    for step in range(40):
        c.append([1, 1])
        c.check_indices()
        c.check_decode(step, f"step {step}")
    c.close()


@pytest.mark.parametrize("dtype,kernel", VARIANTS, ids=IDS)
@pytest.mark.parametrize("S,R", [(16, 112), (0, 5), (64, 256), (3, 1), (30, 37)])
def test_multi_token_and_ragged_appends(gpu_device, dtype, kernel, S, R):
    """Chunks longer than the ring, zero-length chunks, chunks that straddle sink/ring."""
    W = S + R
    c = Case(Hq=8, Hkv=2, B=3, S=S, R=R, dtype=dtype, kernel=kernel, mask=[0, 1], cap=4 * W + 200, seed=5)
    plan = [[1, 0, S + 1], [R + 3, 2, 0], [0, W, 1], [2 * R + 1, 1, R], [5, 3 * R + 7, 40], [1, 1, 1]]
    for i, counts in enumerate(plan):
        c.append(counts)
        c.check_indices()
        if (c.n > 0).all():
            c.check_decode(i, f"chunk {i}")
    c.close()


@pytest.mark.parametrize("dtype,kernel", VARIANTS, ids=IDS)
@pytest.mark.parametrize("Hq,Hkv", [(32, 8), (28, 4), (7, 1)])
def test_fused_append_decode_token_by_token(gpu_device, dtype, kernel, Hq, Hkv):
    """rlkv_append_decode from an empty... almost empty cache: 1 token, then 75 fused steps through the
    sink, the window, two ring wraps, tile boundaries and two work-list rebuilds."""
    mask = [(h % 2) for h in range(Hkv)]
    c = Case(Hq=Hq, Hkv=Hkv, B=2, S=4, R=28, dtype=dtype, kernel=kernel, mask=mask, cap=96, seed=19)
    c.append([1, 3])
    for step in range(75):
        c.check_decode(step, f"fused step {step}", fused=True)
        c.check_indices()
    c.close()


@pytest.mark.parametrize("dtype,kernel", VARIANTS, ids=IDS)
def test_fused_append_decode_long_ragged(gpu_device, dtype, kernel):
    c = Case(Hq=8, Hkv=2, B=3, S=64, R=256, dtype=dtype, kernel=kernel, mask=[1, 0], cap=4200, seed=23)
    c.append([4000, 2017, 319])
    c.check_decode(0, "prefill")
    for step in range(40):
        c.check_decode(step + 1, f"fused step {step}", fused=True)
    c.check_indices()
    c.append([5, 0, 9])            # ragged append invalidates the list: next decode rebuilds it
    c.check_decode(99, "after ragged append")
    c.check_decode(100, "fused again", fused=True)
    c.check_indices()
    c.close()


@pytest.mark.parametrize("dtype,kernel", VARIANTS, ids=IDS)
def test_tile_boundaries(gpu_device, dtype, kernel):
    c = Case(Hq=4, Hkv=1, B=1, S=2, R=3, dtype=dtype, kernel=kernel, mask=[1], cap=200, seed=7)
    n = 0
    for target in [1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 160]:
        c.append([target - n])
        n = target
        c.check_decode(target, f"n={target}")
    c.close()


@pytest.mark.parametrize("dtype,kernel", VARIANTS, ids=IDS)
@pytest.mark.parametrize("mask", [[1, 1], [1, 0], [0, 0]], ids=["allfull", "mixed", "allcomp"])
def test_long_ragged_context_split_over_many_workgroups(gpu_device, dtype, kernel, mask):
    """Several thousand tokens per full head: every pair is cut into many split-K shares."""
    c = Case(Hq=14, Hkv=2, B=3, S=64, R=256, dtype=dtype, kernel=kernel, mask=mask, cap=6100, seed=11)
    c.append([6001, 3333, 517])
    c.check_indices()
    c.check_decode(0, "prefill")
    for step in range(3):
        c.append([1, 1, 1])
        c.check_decode(step + 1, f"step {step}")
    c.check_indices()
    c.close()


@pytest.mark.parametrize("dtype,kernel", VARIANTS, ids=IDS)
def test_deterministic_and_garbage_arena(gpu_device, dtype, kernel):
    """Unwritten store rows hold NaN bit patterns; outputs must not see them, and two runs agree bitwise."""
    c = Case(Hq=8, Hkv=2, B=2, S=8, R=24, dtype=dtype, kernel=kernel, mask=[1, 0], cap=700, seed=13, arena_fill=0xFF)
    c.append([613, 45])
    c.check_decode(0, "garbage arena")
    _, o1 = c.decode(5)
    _, o2 = c.decode(5)
    assert torch.equal(o1.view(torch.int16 if dtype == BF16 else torch.int32),
                       o2.view(torch.int16 if dtype == BF16 else torch.int32))
    c.close()


@pytest.mark.parametrize("dtype,kernel", VARIANTS, ids=IDS)
def test_reset_and_error_paths(gpu_device, dtype, kernel):
    c = Case(Hq=4, Hkv=2, B=2, S=4, R=8, dtype=dtype, kernel=kernel, mask=[1, 0], cap=40, seed=17)
    q = torch.zeros(2, 4, 128, dtype=c.tdtype, device=c.device)
    out = torch.zeros_like(q)
    with pytest.raises(rl.RlkvError) as e:                       # empty cache
        c.cache.decode_attention(0, q, out, 1.0)
    assert e.value.status == binding.RLKV_ERR_STATE
    c.append([30, 30])
    c.check_decode(0, "before reset")
    k = torch.zeros(2, 2, 11, 128, dtype=c.tdtype, device=c.device)
    with pytest.raises(rl.RlkvError) as e:                       # 30 + 11 > 40: nothing is written
        c.cache.append(0, k, k)
    assert e.value.status == binding.RLKV_ERR_CAPACITY
    c.check_indices()
    with pytest.raises(rl.RlkvError) as e:
        c.cache.decode_attention(1, q, out, 1.0)                 # layer out of range
    assert e.value.status == binding.RLKV_ERR_INVALID_ARG
    # reset one sequence: its length and ring slots are empty again, the other is untouched
    c.cache.reset(0)
    c.n[0] = 0
    c.check_indices()
    with pytest.raises(rl.RlkvError) as e:
        c.cache.decode_attention(0, q, out, 1.0)
    assert e.value.status == binding.RLKV_ERR_STATE
    c.append([7, 0])                                             # refill from position 0 (same history rows)
    c.check_indices()
    c.check_decode(1, "after reset + refill")
    c.cache.reset(-1)
    c.n[:] = 0
    c.check_indices()
    c.close()


def test_compressed_store_is_constant_size(gpu_device):
    def resident(max_len, mask):
        cache = rl.Cache(1, 4, 2, 128, 2, 16, 48, BF16, mask, [max_len, max_len])
        r = cache.resident_bytes()
        cache.close()
        return r
    assert resident(64, [0, 0]) == resident(64000, [0, 0]) == 2 * 2 * 2 * 64 * 256
    assert resident(64000, [1, 0]) - resident(64, [1, 0]) == 2 * 2 * (64000 - 64) * 256


def test_auto_kernel_selection(gpu_device):
    a = rl.Cache(1, 4, 2, 128, 1, 4, 4, BF16, [1, 0], [32])
    b = rl.Cache(1, 4, 2, 128, 1, 4, 4, F32, [1, 0], [32])
    assert a.kernel() == MFMA and b.kernel() == VALU
    a.close()
    b.close()


def test_stream_read_probe_runs_and_validates(gpu_device):
    """The measurement aid: launches on any buffer of whole 16 KiB blocks, rejects bad arguments on the host."""
    buf = torch.ones(3 * 16384 // 4 + 5, dtype=torch.int32, device=gpu_device)
    sink = torch.zeros(4, dtype=torch.int32, device=gpu_device)
    for wgs in (1, 7, 256):
        rl.rlkv_probe_stream_read(buf.data_ptr(), buf.numel() * 4, sink.data_ptr(), wgs)
    rl.rlkv_probe_stream_read(buf.data_ptr(), 100, sink.data_ptr(), 4)          # less than one block: nothing to do
    torch.cuda.synchronize()
    assert int(sink.sum()) == 0 and int(buf.sum()) == buf.numel()
    lib = rl.load_library()
    assert lib.rlkv_probe_stream_read(None, 16384, sink.data_ptr(), 4, None) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_probe_stream_read(buf.data_ptr(), 16384, None, 4, None) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_probe_stream_read(buf.data_ptr(), 16384, sink.data_ptr(), 0, None) == binding.RLKV_ERR_INVALID_ARG


@pytest.mark.parametrize("B,Hq,Hkv", [(600, 16, 8), (300, 28, 4)])
def test_many_pairs(gpu_device, B, Hq, Hkv):
    """More (sequence, KV head) pairs than workgroups by far: 4800 pairs take the work list's
    equal-count fallback, 1200 its several scan blocks; ragged short contexts, fused steps, an
    inactive stripe."""
    mask = [(h % 3 != 0) for h in range(Hkv)]
    c = Case(Hq=Hq, Hkv=Hkv, B=B, S=2, R=6, dtype=BF16, kernel=MFMA, mask=mask, cap=48, seed=6)
    rng = np.random.RandomState(B)
    c.append(rng.randint(1, 30, size=B))
    c.check_decode(0, "after the ragged fill")
    active = np.ones(B, dtype=np.uint8)
    active[::7] = 0
    c.cache.set_active(active)
    q, out = c.append_decode(1)
    c.n -= (1 - active).astype(np.int64)               # the harness counted every slot
    import oracle
    from harness import to_np, tolerance
    ref = oracle.decode_attention(to_np(c.k_hist), to_np(c.v_hist), c.n, c.mask_layer, to_np(q), c.S, c.R, c.scale)
    got = out.float().cpu().numpy().astype(np.float64)
    live = active == 1
    assert np.isnan(got[~live]).all()                  # rows of inactive slots keep the harness's NaN fill
    err = np.abs(got[live] - ref[live])
    assert (err <= tolerance(ref[live], BF16)).all(), err.max()
    c.cache.set_active(None)
    for step in range(2, 5):
        c.check_decode(step, f"step {step}", fused=True)
    c.check_indices()
    c.close()


def test_many_pairs_with_a_few_long_sequences(gpu_device):
    """600 pairs (more than the merge kernel takes as arguments: it reads the pair records from memory), three of
    the 150 sequences long enough for their full heads to be split over many workgroups and merged."""
    B = 150
    c = Case(Hq=8, Hkv=4, B=B, S=4, R=28, dtype=BF16, kernel=MFMA, mask=[1, 0, 1, 0], cap=2100, seed=16)
    counts = np.random.RandomState(3).randint(1, 40, size=B)
    counts[[5, 77, 149]] = [2000, 1500, 2047]
    c.append(counts)
    c.check_decode(0, "after the ragged fill")
    for step in range(1, 4):
        c.check_decode(step, f"step {step}", fused=True)
    c.check_indices()
    c.close()


@pytest.mark.parametrize("dtype,kernel", VARIANTS, ids=IDS)
@pytest.mark.parametrize("scale", [-0.07, 0.0])
def test_decode_with_unusual_softmax_scales(gpu_device, dtype, kernel, scale):
    """A negative scale prefers the least similar keys, zero gives uniform weights: both are plain
    softmax attention and must match the oracle like any other scale."""
    c = Case(Hq=28, Hkv=4, B=2, S=4, R=20, dtype=dtype, kernel=kernel, mask=[1, 0, 1, 0], cap=300, seed=43, scale=scale)
    c.append([200, 77])
    for step in range(4):
        c.check_decode(step, f"scale {scale} step {step}", fused=step % 2 == 0)
    c.cache.set_gates(np.array([0.5, 1, 0.2, 1], dtype=np.float32))
    c.check_decode(9, f"scale {scale} gated", gates=[0.5, 1, 0.2, 1])
    c.close()


def test_calls_on_a_side_stream(gpu_device):
    """Every call takes the stream it is given: appends, work-list copies, attention and merge all run
    in order on a non-default stream while the default stream is kept busy with unrelated work."""
    c = Case(Hq=32, Hkv=8, B=2, S=4, R=28, dtype=BF16, kernel=MFMA, mask=[1, 0, 1, 0, 0, 1, 1, 0], cap=400, seed=51,
             prefill_tokens=64)
    side = torch.cuda.Stream()
    noise = torch.ones(1 << 24, device=gpu_device)
    with torch.cuda.stream(side):
        for step in range(3):
            noise.mul_(1.0001)                           # default-stream tensor touched from the side stream too
            c.check_prefill([64, 40], step, f"side-stream chunk {step}")
        for step in range(40):                           # crosses a work-list refresh
            c.check_decode(step, f"side-stream step {step}", fused=step % 4 != 3)
        c.check_indices()
    torch.cuda.synchronize()
    c.close()
