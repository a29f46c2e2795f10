"""Prefill / chunked-prefill attention for mixed heads through the C-ABI (paper Sec. 3.1: causal
mask for full heads, local mask - sink + recent - for compressed heads; App. B: masks applied at
prefill), against the oracle's mask-matrix definition on the complete history.  Every call also
appends its chunk, so lengths, ring slots and a following decode step are checked too."""
import numpy as np
import pytest
import torch

import paper_2510_08525_amd as rl
from paper_2510_08525_amd import binding
import harness
from harness import Case, tolerance

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=["form by size", "two-group form"])
def kernel_form(request, monkeypatch):
    """The library runs a chunk with few long workgroups (most shapes of this file) through the kernel form with
    one column group of queries per wavefront; every test also runs with that choice switched off, so that the
    two-group form sees the same small shapes and edge cases as the full-size workloads give it."""
    monkeypatch.setattr(harness, "TUNING", {"prefill_two_group_only": 1} if request.param == "two-group form" else {})
    yield request.param

MFMA, BF16 = rl.RLKV_KERNEL_MFMA, rl.RLKV_BF16
SHAPES = [(32, 8, [1, 0, 1, 1, 0, 0, 1, 0]), (28, 4, [1, 0, 0, 1]), (8, 8, [0, 1, 0, 1, 1, 0, 0, 1]), (16, 1, [0]),
          (7, 1, [1]), (12, 4, [0, 0, 1, 0])]


@pytest.mark.parametrize("Hq,Hkv,mask", SHAPES, ids=[f"{a}q{b}kv" for a, b, _ in SHAPES])
@pytest.mark.parametrize("S,R", [(4, 24), (16, 112), (0, 5), (33, 70), (3, 1)])
def test_chunked_prefill_matches_mask_matrices(gpu_device, Hq, Hkv, mask, S, R):
    """Chunks longer and shorter than the ring, ragged counts, an idle sequence, a one-token chunk."""
    c = Case(Hq=Hq, Hkv=Hkv, B=3, S=S, R=R, dtype=BF16, kernel=MFMA, mask=mask, cap=700, seed=21,
             prefill_tokens=256, arena_fill=0xFF)
    worst = 0.0
    for step, counts in enumerate([[200, 37, 0], [256, 1, 90], [3, 0, 129], [64, 64, 64]]):
        worst = max(worst, c.check_prefill(counts, step, f"chunk {step}"))
        c.check_indices()
    c.check_decode(0, "decode after the prefill", fused=True)
    worst = max(worst, c.check_prefill([30, 100, 7], 9, "chunk after a decode step"))
    c.check_indices()
    c.check_decode(1, "decode after the second prefill")
    print("worst abs err", worst)
    c.close()


def test_prefill_first_chunk_equals_plain_causal_attention(gpu_device):
    """Every head full, empty cache: the textbook causal prefill, against the library routine."""
    Hq, Hkv, B, T, D = 8, 2, 2, 160, 128
    c = Case(Hq=Hq, Hkv=Hkv, B=B, S=4, R=8, dtype=BF16, kernel=MFMA, mask=[1, 1], cap=T, seed=5, prefill_tokens=T,
             sink_keys=False)
    from inputs import synth
    q = synth.normal(5, synth.T_Q, 0, range(B), range(Hq), 0, T, D, dtype=torch.bfloat16)
    out = torch.zeros(B, Hq, T, D, dtype=torch.bfloat16, device=c.device)
    c.cache.prefill_attention(0, q.to(c.device), c.k_hist.to(c.device), c.v_hist.to(c.device), [T, T], out, c.scale)
    torch.cuda.synchronize()
    kk = c.k_hist.double().repeat_interleave(Hq // Hkv, dim=1)
    vv = c.v_hist.double().repeat_interleave(Hq // Hkv, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(q.double(), kk, vv, is_causal=True, scale=c.scale)
    err = (out.cpu().double() - ref).abs().numpy()
    assert (err <= tolerance(ref.numpy(), BF16)).all(), err.max()
    c.close()


@pytest.mark.parametrize("page", [32, 128])
def test_prefill_over_paged_full_heads(gpu_device, page):
    c = Case(Hq=28, Hkv=4, B=2, S=8, R=40, dtype=BF16, kernel=MFMA, mask=[1, 0, 1, 1], cap=600, seed=8,
             prefill_tokens=192, page_tokens=page, pool_pages=2 * (-(-600 // page)))
    c.cache.pool_shuffle(3)
    for step, counts in enumerate([[192, 50], [100, 192], [150, 31]]):
        c.check_prefill(counts, step, f"paged chunk {step}")
    c.check_indices()
    for step in range(5):
        c.check_decode(step, f"decode {step}", fused=True)
    c.close()


def test_prefill_with_stride_longer_than_the_counts(gpu_device):
    c = Case(Hq=32, Hkv=8, B=2, S=4, R=12, dtype=BF16, kernel=MFMA, mask=[1, 0] * 4, cap=300, seed=2, prefill_tokens=128)
    c.check_prefill([40, 9], 0, "stride 128, short counts", stride=128)
    c.check_prefill([0, 0], 1, "nothing to do", stride=16)
    c.check_prefill([1, 127], 2, "one token and a long one", stride=128)
    c.check_indices()
    c.close()


def test_prefill_error_paths(gpu_device):
    dev = torch.device("cuda:0")
    kw = dict(Hq=8, Hkv=2, B=2, S=4, R=8, dtype=BF16, kernel=MFMA, mask=[1, 0], cap=100, seed=1)
    no = Case(**kw)                                       # created without a staging buffer
    q = torch.zeros(2, 8, 16, 128, dtype=torch.bfloat16, device=dev)
    k = torch.zeros(2, 2, 16, 128, dtype=torch.bfloat16, device=dev)
    out = torch.full_like(q, 3.0)
    with pytest.raises(rl.RlkvError) as e:
        no.cache.prefill_attention(0, q, k, k, [16, 16], out, 1.0)
    assert e.value.status == binding.RLKV_ERR_STATE
    no.close()
    c = Case(prefill_tokens=16, **kw)
    q32 = torch.zeros(2, 8, 32, 128, dtype=torch.bfloat16, device=dev)
    k32 = torch.zeros(2, 2, 32, 128, dtype=torch.bfloat16, device=dev)
    with pytest.raises(rl.RlkvError) as e:                # chunk longer than the staging buffer
        c.cache.prefill_attention(0, q32, k32, k32, [32, 1], torch.zeros_like(q32), 1.0)
    assert e.value.status == binding.RLKV_ERR_INVALID_ARG
    with pytest.raises(rl.RlkvError) as e:                # count above the stride
        c.cache.prefill_attention(0, q, k, k, [17, 1], out, 1.0)
    assert e.value.status == binding.RLKV_ERR_INVALID_ARG
    c.append([90, 10])
    with pytest.raises(rl.RlkvError) as e:                # 90 + 16 > max_len: nothing computed, nothing appended
        c.cache.prefill_attention(0, q, k, k, [16, 16], out, 1.0)
    assert e.value.status == binding.RLKV_ERR_CAPACITY
    torch.cuda.synchronize()
    assert (out.float() == 3.0).all()
    c.check_indices()
    c.check_prefill([5, 16], 0, "after the refused calls")
    c.close()


@pytest.mark.parametrize("Hq,Hkv,mask,gates", [
    (32, 8, [1, 0, 1, 1, 0, 0, 1, 1], [0.3, 1, 0.0, 1.0, 1, 1, 0.75, 0.5]),
    (28, 4, [1, 1, 1, 1], [0.25, 0.6, 0.0, 0.9]),
    (16, 1, [1], [0.4]),
])
@pytest.mark.parametrize("S,R", [(4, 24), (33, 70), (0, 5)])
def test_gated_prefill_blends_causal_and_local(gpu_device, Hq, Hkv, mask, gates, S, R):
    """Eq. 1 at prefill (the prompt of a rollout): gate * causal + (1 - gate) * local per full head,
    chunk after chunk, with decode steps in between; compressed heads keep the local mask."""
    c = Case(Hq=Hq, Hkv=Hkv, B=3, S=S, R=R, dtype=BF16, kernel=MFMA, mask=mask, cap=900, seed=33, prefill_tokens=256)
    g = np.asarray(gates, dtype=np.float32)
    c.cache.set_gates(g)
    for step, counts in enumerate([[200, 37, 0], [256, 1, 90], [130, 256, 129], [64, 64, 64]]):
        c.check_prefill(counts, step, f"gated chunk {step}", gates=g)
        c.check_indices()
    c.check_decode(0, "gated decode after the prefill", fused=True, gates=g)
    c.check_prefill([17, 100, 3], 7, "gated chunk after a decode step", gates=g)
    c.cache.set_gates(None)
    c.check_prefill([50, 50, 50], 8, "gates back to 1")
    c.close()


def test_prefill_addresses_the_right_layer(gpu_device):
    """A three-layer cache whose layers differ in mask and gates: prefill and decode on layer 1 only."""
    c = Case(Hq=28, Hkv=4, B=2, S=8, R=24, dtype=BF16, kernel=MFMA, mask=[0, 1, 1, 0], cap=500, seed=17,
             n_layers=3, layer=1, prefill_tokens=128)
    g = np.ones((3, 4), dtype=np.float32)
    g[1] = [1, 0.5, 1, 1]
    g[0] = g[2] = 0.0                                   # other layers' gates must not leak in
    c.cache.set_gates(g.reshape(-1))
    c.check_prefill([128, 77], 0, "layer 1, chunk 0", gates=g[1])
    c.check_prefill([100, 128], 1, "layer 1, chunk 1", gates=g[1])
    c.check_indices()
    c.check_decode(0, "layer 1 decode", fused=True, gates=g[1])
    assert c.cache.lengths(0).tolist() == [0, 0] and c.cache.lengths(2).tolist() == [0, 0]
    c.close()


@pytest.mark.parametrize("scale", [-0.07, 0.0, 0.31])
def test_prefill_with_unusual_softmax_scales(gpu_device, scale):
    """A negative scale (the running maximum would become a minimum: the kernel takes its general
    loop throughout), zero (uniform weights) and a large one."""
    c = Case(Hq=28, Hkv=4, B=2, S=4, R=20, dtype=BF16, kernel=MFMA, mask=[1, 0, 1, 0], cap=400, seed=41,
             prefill_tokens=128, scale=scale)
    c.check_prefill([128, 60], 0, f"scale {scale} chunk 0")
    c.check_prefill([100, 128], 1, f"scale {scale} chunk 1")
    c.check_decode(0, f"scale {scale} decode", fused=True)
    c.close()


@pytest.mark.parametrize("prescale", [6.0, 25.0])
def test_prefill_with_peaked_scores(gpu_device, prescale):
    """Large scores: the softmax is nearly one-hot and the running maxima jump by far more than the
    slack that lets the kernel postpone its rescaling; full and gated heads, hot and general loop."""
    c = Case(Hq=32, Hkv=8, B=2, S=8, R=40, dtype=BF16, kernel=MFMA, mask=[1, 0, 1, 1, 0, 1, 1, 0], cap=900, seed=47,
             prefill_tokens=256, q_prescale=prescale)
    c.check_prefill([256, 100], 0, "chunk 0")
    c.check_prefill([256, 256], 1, "chunk 1")
    g = np.array([0.5, 1, 1, 0.1, 1, 1, 0.9, 1], dtype=np.float32)
    c.cache.set_gates(g)
    c.check_prefill([200, 256], 2, "gated chunk", gates=g)
    c.check_decode(0, "decode", fused=True, gates=g)
    c.close()


def test_prefill_is_deterministic_and_layout_independent(gpu_device):
    """The same chunks through three caches - contiguous, contiguous again (arena pre-filled with a
    different byte pattern), paged with a shuffled pool - give bit-identical outputs: the order of
    accumulation is fixed by the work split, not by timing or by where the rows live."""
    kw = dict(Hq=28, Hkv=4, B=2, S=8, R=40, dtype=BF16, kernel=MFMA, mask=[1, 0, 1, 1], cap=700, seed=61, prefill_tokens=256)
    a = Case(arena_fill=0x00, **kw)
    b = Case(arena_fill=0xFF, **kw)
    p = Case(page_tokens=64, pool_pages=24, **kw)
    p.cache.pool_shuffle(9)
    g = np.array([0.6, 1, 1, 0.2], dtype=np.float32)
    for step, counts in enumerate([[256, 100], [200, 256], [77, 1]]):
        if step == 2:
            for c in (a, b, p):
                c.cache.set_gates(g)
        outs = []
        for c in (a, b, p):
            c.check_prefill(counts, step, f"chunk {step}", gates=g if step == 2 else None)
            outs.append(c.last_out.cpu().view(torch.int16))
        assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2]), f"chunk {step}"
    for c in (a, b, p):
        c.close()


def test_prefill_with_values_beyond_the_fp16_range(gpu_device):
    """The kernel takes V through fp16 operands where it can; once a value of magnitude 65536 or more
    has gone into a layer it must take V as the stored bf16 bits.  A sink position, one more cached position and one
    position of a later chunk carry |V| scaled by 1e5 (one sign, so that no output is the small difference of two
    huge terms); the tiles around them are ordinary.  Outputs reach 1e5, where
    the final bf16 rounding alone uses up the half ulp the tolerance grants: 2^-10 |ref| more for the
    error before it (the 1e-2 of unit-scale V, scaled)."""
    c = Case(Hq=28, Hkv=4, B=2, S=8, R=40, dtype=BF16, kernel=MFMA, mask=[1, 0, 1, 1], cap=800, seed=77,
             prefill_tokens=256)
    for pos in (5, 70, 300):
        c.v_hist[:, :, pos] = (c.v_hist[:, :, pos].float().abs() * 1e5).to(torch.bfloat16)
    assert c.v_hist.float().abs().max() > 65536
    for step, counts in enumerate([[256, 200], [256, 256], [100, 256]]):
        c.check_prefill(counts, step, f"chunk {step}", rel=2.0 ** -10)
    c.check_decode(0, "decode", fused=True, rel=2.0 ** -10)
    c.close()


@pytest.mark.parametrize("how", ["fused step", "ragged append", "uniform append"])
def test_prefill_after_a_wide_value_arrived_by_another_call(gpu_device, how):
    """The value beyond the fp16 range reaches the store through a decode step's fused append or through
    a plain append, not through a prefill chunk; the next chunk reads it from the store."""
    c = Case(Hq=28, Hkv=4, B=2, S=8, R=40, dtype=BF16, kernel=MFMA, mask=[1, 0, 1, 1], cap=900, seed=78,
             prefill_tokens=256)
    c.check_prefill([256, 256], 0, "ordinary chunk")
    pos = 256 if how == "fused step" else 259
    c.v_hist[:, :, pos] = (c.v_hist[:, :, pos].float().abs() * 1e5).to(torch.bfloat16)
    if how == "fused step":
        c.check_decode(0, "the step that brings the value", fused=True, rel=2.0 ** -10)
    elif how == "ragged append":
        c.append([10, 4])
    else:
        c.append([6, 6])
    c.check_prefill([256, 200], 1, "chunk over the store", rel=2.0 ** -10)
    c.check_decode(1, "decode", fused=True, rel=2.0 ** -10)
    # emptied as a whole, the cache starts over (ordinary values only from here on)
    c.cache.reset()
    c.n[:] = 0
    c.v_hist[:, :, pos] = (c.v_hist[:, :, pos].float() * 1e-5).to(torch.bfloat16)
    c.check_prefill([256, 256], 2, "after the reset")
    c.check_prefill([256, 256], 3, "after the reset, second chunk")
    c.close()


@pytest.mark.parametrize("value", [65280.0, 65536.0, -65536.0, 2.0 ** -15, 2.0 ** -26])
def test_prefill_at_the_edges_of_the_fp16_range(gpu_device, value):
    """65280 is the largest bf16 value below 65536 and still an fp16 value; 65536 is the first one
    that is not (it must switch the layer to bf16 operands); 2^-15 becomes an fp16 subnormal
    exactly; 2^-26 is lost on the fp16 road, which the absolute bar does not see.  A whole row of
    one KV head carries the value."""
    c = Case(Hq=28, Hkv=4, B=2, S=8, R=40, dtype=BF16, kernel=MFMA, mask=[1, 0, 1, 1], cap=600, seed=79,
             prefill_tokens=256)
    c.v_hist[:, 0, 33] = value
    c.check_prefill([256, 256], 0, "first chunk", rel=2.0 ** -10)
    c.check_prefill([200, 256], 1, "chunk over the store", rel=2.0 ** -10)
    c.close()


@pytest.mark.parametrize("Hq,Hkv,mask,S,R", [(28, 4, [1, 0, 0, 1], 64, 256), (16, 4, [0, 0, 1, 0], 32, 96),
                                              (8, 8, [0, 1, 0, 0, 1, 0, 0, 0], 48, 300), (16, 1, [0], 0, 64)],
                         ids=["7x-64-256", "4x-32-96", "1x-48-300", "16x-0-64"])
def test_prefill_with_chunks_longer_than_the_recent_band(gpu_device, Hq, Hkv, mask, S, R):
    """Chunks of several hundred tokens against a shorter band: most of what a compressed head attends
    over then lies in chunk tiles that every query of a workgroup sees whole, next to its complete
    sink tiles in the store (S = 48: one complete, one partial; S = 0: none)."""
    c = Case(Hq=Hq, Hkv=Hkv, B=2, S=S, R=R, dtype=BF16, kernel=MFMA, mask=mask, cap=1800, seed=31,
             prefill_tokens=512, arena_fill=0xFF)
    for step, counts in enumerate([[512, 300], [512, 512], [300, 77]]):
        c.check_prefill(counts, step, f"chunk {step}")
        c.check_indices()
    c.check_decode(0, "decode after the prefill", fused=True)
    c.check_prefill([100, 512], 5, "chunk after a decode step")
    c.check_indices()
    # the same heads in the kernel form for blending layers (one column group per wavefront)
    g = np.where(np.asarray(mask) == 1, 0.25, 1.0).astype(np.float32)
    c.cache.set_gates(g)
    c.check_prefill([256, 100], 6, "chunk in a blending layer", gates=g)
    c.close()


@pytest.mark.parametrize("seed", range(12))
def test_prefill_random_windows_chunks_and_gates(gpu_device, seed):
    """Drawn per seed: head shape, mask, sink and band sizes around and above a tile and a workgroup's
    span, chunk lengths (full, partial, empty), gates in a third of the cases, decode steps between."""
    rng = np.random.default_rng(1000 + seed)
    Hq, Hkv = [(32, 8), (28, 4), (8, 8), (7, 1), (16, 1), (12, 4), (10, 2)][rng.integers(7)]
    S = int(rng.choice([0, 16, 32, 48, 64, 96]))
    R = int(rng.choice([33, 64, 100, 128, 256, 300]))
    T = int(rng.choice([256, 512]))
    mask = rng.integers(0, 2, size=Hkv).tolist()
    c = Case(Hq=Hq, Hkv=Hkv, B=2, S=S, R=R, dtype=BF16, kernel=MFMA, mask=mask, cap=4 * T + 8, seed=seed,
             prefill_tokens=T, arena_fill=0xFF)
    g = None
    if rng.random() < 0.3:
        g = rng.choice([0.0, 0.3, 1.0], size=Hkv).astype(np.float32)
        c.cache.set_gates(g)
    for step in range(4):
        counts = [int(rng.choice([T, T, int(rng.integers(0, T + 1))])) for _ in range(2)]
        c.check_prefill(counts, step, f"seed {seed} chunk {step} (S {S} R {R} T {T} mask {mask} gates {g})", gates=g)
        if rng.random() < 0.3:
            c.check_decode(step, f"seed {seed} decode {step}", fused=True, gates=g)
    c.check_indices()
    c.close()


@pytest.mark.parametrize("B,mask", [(1, [1, 0, 0, 1]), (1, [0, 0, 1, 0]), (2, [1, 0, 1, 1])], ids=["1seq-2full", "1seq-1full", "2seq-3full"])
def test_prefill_of_few_long_sequences(gpu_device, B, mask, monkeypatch):
    """One or two sequences with a few full heads give fewer long workgroups than the chip has compute
    units: once the cached context is long enough the library divides each one's tiles among several
    workgroups and merges their shares.  The library's threshold (80 tiles per share) is lowered here so
    that 2, 4 and 8 shares occur as this small context grows.  Ragged counts and a paged variant of
    the same sizes included."""
    monkeypatch.setattr(harness, "TUNING", dict(harness.TUNING, prefill_min_share_tiles=8))
    for page in (0, 64):
        c = Case(Hq=28, Hkv=4, B=B, S=32, R=96, dtype=BF16, kernel=MFMA, mask=mask, cap=4700, seed=41 + B,
                 prefill_tokens=512, page_tokens=page, pool_pages=B * 74 if page else 0)
        if page:
            c.cache.pool_shuffle(5)
        for step in range(8):
            counts = [512] * B if step != 5 else [300] + [512] * (B - 1)
            c.check_prefill(counts, step, f"page {page} chunk {step}")
        c.check_indices()
        c.check_decode(0, "decode after the prefill", fused=True)
        c.check_prefill([77] * B, 9, "a short chunk over a long context")
        c.close()


def test_prefill_of_one_long_sequence_at_the_default_threshold(gpu_device):
    """6000 cached positions (plain appends), then chunks of 512: with one sequence and two full heads
    each workgroup's 187 unmasked tiles go to two workgroups."""
    c = Case(Hq=28, Hkv=4, B=1, S=64, R=256, dtype=BF16, kernel=MFMA, mask=[1, 0, 0, 1], cap=7100, seed=47,
             prefill_tokens=512)
    for _ in range(3):
        c.append([2000])
    c.check_prefill([512], 0, "first chunk over 6000 positions")
    c.check_prefill([400], 1, "second chunk")
    c.check_indices()
    c.check_decode(0, "decode after the prefill", fused=True)
    c.close()


def test_prefill_with_more_kv_heads_than_the_kernel_arguments_list(gpu_device):
    """72 KV heads: the lists of full and compressed heads no longer fit the kernel's arguments (64) and
    every workgroup finds its head from the layer's mask in memory."""
    mask = [(h * 7) % 3 != 0 for h in range(72)]
    c = Case(Hq=72, Hkv=72, B=2, S=4, R=40, dtype=BF16, kernel=MFMA, mask=mask, cap=400, seed=72, prefill_tokens=128)
    c.check_prefill([128, 50], 0, "chunk 0")
    c.check_prefill([100, 128], 1, "chunk 1")
    c.check_indices()
    c.check_decode(0, "decode", fused=True)
    c.close()


@pytest.mark.parametrize("B,Hq,Hkv,mask", [(5, 12, 3, [1, 1, 0]), (9, 8, 2, [1, 0]), (6, 8, 8, [1, 1, 1, 0, 1, 1, 1, 1]),
                                           (17, 4, 1, [1]), (8, 4, 2, [0, 0]), (37, 8, 8, [1, 0, 1, 1, 0, 0, 1, 1])],
                         ids=["10heavy-15rows", "9heavy-18rows", "42heavy-48rows", "17heavy-17rows", "0heavy-16rows",
                              "185heavy-296rows"])
def test_prefill_grid_rows_dealt_to_xcds(gpu_device, B, Hq, Hkv, mask):
    """Row counts that are no multiples of 8 in either class: equal chunks (the leading groups of 8 full-head rows
    go one row per XCD, the rest workgroup by workgroup), then a ragged chunk with idle sequences (fewer rows
    dealt by rows, or none); every output row of every sequence is compared, so a workgroup dealt twice or not at
    all would show."""
    T = 160
    c = Case(Hq=Hq, Hkv=Hkv, B=B, S=8, R=40, dtype=BF16, kernel=MFMA, mask=mask, cap=3 * T + 4, seed=77,
             prefill_tokens=T, arena_fill=0xFF)
    n_full = int(sum(mask))
    assert rl.rlkv_plan_prefill_rows(n_full, [T] * B, [0] * B) == (8 * (B * n_full // 8), B * n_full)
    c.check_prefill([T] * B, 0, "equal chunks")
    c.check_prefill([T] * B, 1, "equal chunks over cached context")
    ragged = [T if b % 3 == 0 else (0 if b % 3 == 1 else 17 + b) for b in range(B)]
    c.check_prefill(ragged, 2, "ragged chunk")
    c.check_indices()
    c.check_decode(0, "decode after the prefill", fused=True)
    c.close()
