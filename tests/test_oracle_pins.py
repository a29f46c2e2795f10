"""Pins of the CPU oracle to things other than itself.

Each test checks oracle/rlkv_oracle.c against a library routine, a closed form, an
invariant or an independent brute force, so that a dropped term, a wrong sign or index,
or a transposed operand in the oracle fails at least one of them.  CPU only.
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from inputs import synth, workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(seed, B, Hq, Hkv, cap, D, dtype=torch.float32):
    k = synth.normal(seed, synth.T_K, 0, range(B), range(Hkv), 0, cap, D, dtype=dtype)
    v = synth.normal(seed, synth.T_V, 0, range(B), range(Hkv), 0, cap, D, dtype=dtype)
    q = synth.normal(seed, synth.T_Q, 0, range(B), range(Hq), 0, 1, D, dtype=dtype)[:, :, 0, :]
    return k, v, q


def _np(t):
    return synth.bf16_bits(t) if t.dtype == torch.bfloat16 else t.numpy()


def _sdpa_rows(k, v, q, rows, scale, G):
    """Library attention (torch SDPA, float64) of every query head over the given rows."""
    Hq = q.shape[0]
    kk = k.double()[:, rows, :].repeat_interleave(G, dim=0)       # [Hq, len(rows), D]
    vv = v.double()[:, rows, :].repeat_interleave(G, dim=0)
    qq = q.double()[:, None, :]                                    # [Hq, 1, D]
    o = torch.nn.functional.scaled_dot_product_attention(qq[None], kk[None], vv[None], scale=scale)
    return o[0, :, 0, :].numpy()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (7, 1), (4, 4)])
def test_all_full_equals_library_attention(dtype, Hq, Hkv):
    B, cap, D = 3, 150, 64
    k, v, q = _rand(11, B, Hq, Hkv, cap, D, dtype)
    n = [150, 97, 1]
    scale = 0.37
    out = oracle.decode_attention(_np(k), _np(v), n, [1] * Hkv, _np(q), 4, 8, scale)
    for b in range(B):
        ref = _sdpa_rows(k[b], v[b], q[b], list(range(n[b])), scale, Hq // Hkv)
        np.testing.assert_allclose(out[b], ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("S,R", [(4, 8), (0, 5), (16, 112), (3, 1)])
def test_compressed_equals_library_attention_over_retained_rows(S, R):
    """Explicit gather of the sink + recent rows, then the library routine."""
    B, Hq, Hkv, cap, D = 4, 6, 3, 300, 32
    k, v, q = _rand(12, B, Hq, Hkv, cap, D)
    n = [300, S + R + 1, S + R + 17, 2 * (S + R) + 5]
    mask = [0, 1, 0]
    out = oracle.decode_attention(_np(k), _np(v), n, mask, _np(q), S, R, 0.25)
    G = Hq // Hkv
    for b in range(B):
        rows_c = [j for j in range(n[b]) if j < S or j >= n[b] - R]
        assert len(rows_c) == min(n[b], S + R)
        ref_c = _sdpa_rows(k[b], v[b], q[b], rows_c, 0.25, G)
        ref_f = _sdpa_rows(k[b], v[b], q[b], list(range(n[b])), 0.25, G)
        for i in range(Hq):
            ref = ref_f if mask[i // G] else ref_c
            np.testing.assert_allclose(out[b, i], ref[i], rtol=0, atol=1e-12)
        # the compressed heads really differ from full once something is evicted
        assert np.abs(ref_c[0] - ref_f[0]).max() > 1e-6


@pytest.mark.parametrize("S,R", [(4, 8), (16, 112), (0, 3)])
def test_compressed_equals_full_until_window_overflows(S, R):
    B, Hq, Hkv, D = 4, 4, 2, 16
    cap = S + R + 2
    k, v, q = _rand(13, B, Hq, Hkv, cap, D)
    lens = [1, max(1, S), S + R - 1 if S + R > 1 else 1, S + R]
    o_full = oracle.decode_attention(_np(k), _np(v), lens, [1, 1], _np(q), S, R, 1.0)
    o_comp = oracle.decode_attention(_np(k), _np(v), lens, [0, 0], _np(q), S, R, 1.0)
    assert np.array_equal(o_full, o_comp)
    lens2 = [S + R + 1] * B          # one eviction: no longer equal
    o_full = oracle.decode_attention(_np(k), _np(v), lens2, [1, 1], _np(q), S, R, 1.0)
    o_comp = oracle.decode_attention(_np(k), _np(v), lens2, [0, 0], _np(q), S, R, 1.0)
    assert np.abs(o_full - o_comp).max() > 1e-6


def test_zero_keys_give_mean_of_position_set_closed_form():
    """K = 0 -> uniform weights; with v_j[d] = j the output is the mean position."""
    S, R, D = 5, 9, 8
    for n in [1, 5, 14, 15, 40, 1000]:
        k = np.zeros((1, 1, n, D), dtype=np.float32)
        v = np.broadcast_to(np.arange(n, dtype=np.float32)[None, None, :, None], (1, 1, n, D)).copy()
        q = np.ones((1, 2, D), dtype=np.float32)
        o_c = oracle.decode_attention(k, v, [n], [0], q, S, R, 1.0)
        o_f = oracle.decode_attention(k, v, [n], [1], q, S, R, 1.0)
        full_mean = (n - 1) / 2.0
        if n <= S + R:
            comp_mean = full_mean
        else:
            comp_mean = (S * (S - 1) / 2.0 + (R * (2 * n - R - 1)) / 2.0) / (S + R)
        np.testing.assert_allclose(o_f, full_mean, rtol=1e-13)
        np.testing.assert_allclose(o_c, comp_mean, rtol=1e-13)


def test_dominating_key_at_evicted_vs_retained_position():
    S, R, D, n = 4, 8, 16, 64
    k, v, q = _rand(14, 1, 2, 2, n, D)
    k, v, q = k.clone(), v.clone(), q.clone()
    q[0, 1] = q[0, 0]                       # both query heads (one per KV head) identical
    k[0, 1] = k[0, 0]
    v[0, 1] = v[0, 0]
    base = oracle.decode_attention(_np(k), _np(v), [n], [1, 0], _np(q), S, R, 1.0)
    for pos, retained in [(S, False), (n - R - 1, False), (20, False),
                          (0, True), (S - 1, True), (n - R, True), (n - 1, True)]:
        kk = k.clone()
        kk[0, :, pos, :] = 50.0 * q[0, 0]   # score ~ 50 |q|^2: dominates the softmax
        out = oracle.decode_attention(_np(kk), _np(v), [n], [1, 0], _np(q), S, R, 1.0)
        np.testing.assert_allclose(out[0, 0], v[0, 0, pos].double().numpy(), atol=1e-9)   # full head
        if retained:
            np.testing.assert_allclose(out[0, 1], v[0, 1, pos].double().numpy(), atol=1e-9)
        else:
            assert np.array_equal(out[0, 1], base[0, 1])   # evicted: compressed head unchanged


def test_weights_are_a_distribution_on_the_position_set():
    S, R = 3, 6
    B, Hq, Hkv, cap, D = 2, 4, 2, 50, 16
    k, v, q = _rand(15, B, Hq, Hkv, cap, D)
    n = [50, 23]
    mask = [1, 0]
    out, w = oracle.decode_attention(_np(k), _np(v), n, mask, _np(q), S, R, 0.5, return_weights=True)
    assert (w >= 0).all()
    np.testing.assert_allclose(w.sum(-1), 1.0, rtol=1e-13)
    for b in range(B):
        for i in range(Hq):
            h = i // 2
            for j in range(cap):
                inside = j < n[b] and (mask[h] or j < S or j >= n[b] - R)
                assert (w[b, i, j] > 0) == inside
                assert oracle.in_position_set(mask[h], j, n[b], S, R) == inside
            np.testing.assert_allclose(out[b, i], w[b, i, :] @ v[b, h].double().numpy(), atol=1e-13)
            lo = v[b, h, :n[b]].double().numpy().min(0)
            hi = v[b, h, :n[b]].double().numpy().max(0)
            assert (out[b, i] >= lo - 1e-12).all() and (out[b, i] <= hi + 1e-12).all()


def test_pure_python_brute_force_tiny():
    S, R, D, n = 2, 3, 4, 9
    k, v, q = _rand(16, 1, 2, 1, n, D)
    scale = 0.7
    out = oracle.decode_attention(_np(k), _np(v), [n], [0], _np(q), S, R, scale)
    for i in range(2):
        keep = [j for j in range(n) if j < S or j >= n - R]
        sc = [scale * sum(float(q[0, i, d]) * float(k[0, 0, j, d]) for d in range(D)) for j in keep]
        mx = max(sc)
        ws = [math.exp(s - mx) for s in sc]
        Z = sum(ws)
        for d in range(D):
            ref = sum(w * float(v[0, 0, j, d]) for w, j in zip(ws, keep)) / Z
            assert abs(out[0, i, d] - ref) < 1e-13


def test_constant_v_and_score_shift_invariance():
    B, Hq, Hkv, cap, D = 1, 2, 1, 40, 8
    k, v, q = _rand(17, B, Hq, Hkv, cap, D)
    vc = torch.full_like(v, 2.5)
    out = oracle.decode_attention(_np(k), _np(vc), [40], [0], _np(q), 4, 8, 1.0)
    np.testing.assert_allclose(out, 2.5, rtol=1e-14)
    # adding a multiple of q's orthogonal complement to all keys: adding the same vector
    # u to every key shifts every score by scale*q.u and must not change the output
    u = torch.randn(D, generator=torch.Generator().manual_seed(1))
    o1 = oracle.decode_attention(_np(k), _np(v), [40], [1], _np(q), 4, 8, 1.0)
    o2 = oracle.decode_attention(_np(k + u), _np(v), [40], [1], _np(q), 4, 8, 1.0)
    np.testing.assert_allclose(o1, o2, atol=1e-5)   # fp32 rounding of k+u only


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (7, 1), (28, 4), (32, 8)])
def test_gqa_head_mapping(Hq, Hkv):
    """V of KV head h is the constant h: query head i must return i // G exactly."""
    D, n = 8, 12
    k, _, q = _rand(18, 1, Hq, Hkv, n, D)
    v = torch.zeros(1, Hkv, n, D)
    for h in range(Hkv):
        v[0, h] = float(h)
    out = oracle.decode_attention(_np(k), _np(v), [n], [h % 2 for h in range(Hkv)], _np(q), 2, 4, 1.0)
    G = Hq // Hkv
    for i in range(Hq):
        np.testing.assert_allclose(out[0, i], float(i // G), atol=1e-14)


def test_f32_variant_tracks_f64():
    B, Hq, Hkv, cap, D = 2, 8, 2, 600, 128
    k, v, q = _rand(19, B, Hq, Hkv, cap, D, torch.bfloat16)
    a = oracle.decode_attention(_np(k), _np(v), [600, 333], [1, 0], _np(q), 16, 64, 1 / math.sqrt(D))
    b = oracle.decode_attention(_np(k), _np(v), [600, 333], [1, 0], _np(q), 16, 64, 1 / math.sqrt(D),
                                precision="f32")
    assert b.dtype == np.float32
    assert np.abs(a - b).max() < 2e-6


def test_invalid_arguments_rejected():
    k = np.zeros((1, 2, 4, 8), dtype=np.float32)
    q = np.zeros((1, 4, 8), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.decode_attention(k, k, [5], [1, 1], q, 1, 1, 1.0)      # n > cap
    with pytest.raises(ValueError):
        oracle.decode_attention(k, k, [0], [1, 1], q, 1, 1, 1.0)      # empty cache
    with pytest.raises(ValueError):
        oracle.decode_attention(k, k, [4], [1, 1], q, 1, 0, 1.0)      # recent < 1


# ---------------------------------------------------------------- Eq. 1 gated mixture

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_gated_mixture_is_the_blend_of_two_library_attentions(dtype):
    B, Hq, Hkv, cap, D, S, R = 2, 6, 3, 90, 32, 4, 10
    k, v, q = _rand(21, B, Hq, Hkv, cap, D, dtype)
    n = [90, 37]
    gate = [1.0, 0.0, 0.3]
    out = oracle.decode_attention_gated(_np(k), _np(v), n, gate, _np(q), S, R, 0.2)
    G = Hq // Hkv
    for b in range(B):
        rows_local = [j for j in range(n[b]) if j < S or j >= n[b] - R]
        full = _sdpa_rows(k[b], v[b], q[b], list(range(n[b])), 0.2, G)
        local = _sdpa_rows(k[b], v[b], q[b], rows_local, 0.2, G)
        for i in range(Hq):
            a = gate[i // G]
            np.testing.assert_allclose(out[b, i], a * full[i] + (1 - a) * local[i], rtol=0, atol=1e-12)
    # gate 1 / gate 0 are the binary head kinds of the inference path
    o1 = oracle.decode_attention_gated(_np(k), _np(v), n, [1, 1, 1], _np(q), S, R, 0.2)
    o0 = oracle.decode_attention_gated(_np(k), _np(v), n, [0, 0, 0], _np(q), S, R, 0.2)
    np.testing.assert_allclose(o1, oracle.decode_attention(_np(k), _np(v), n, [1, 1, 1], _np(q), S, R, 0.2), atol=1e-15)
    np.testing.assert_allclose(o0, oracle.decode_attention(_np(k), _np(v), n, [0, 0, 0], _np(q), S, R, 0.2), atol=1e-15)
    # linear in the gate; no effect while nothing would be evicted (n <= S + R)
    oh = oracle.decode_attention_gated(_np(k), _np(v), n, [0.5] * 3, _np(q), S, R, 0.2)
    np.testing.assert_allclose(oh, 0.5 * (o1 + o0), atol=1e-14)
    short = [S + R, 3]
    a = oracle.decode_attention_gated(_np(k), _np(v), short, [0.25] * 3, _np(q), S, R, 0.2)
    b_ = oracle.decode_attention(_np(k), _np(v), short, [1, 1, 1], _np(q), S, R, 0.2)
    np.testing.assert_allclose(a, b_, atol=1e-14)
    with pytest.raises(ValueError):
        oracle.decode_attention_gated(_np(k), _np(v), n, [1.5, 0, 0], _np(q), S, R, 0.2)


def test_gated_f32_variant_is_pinned_to_library_attention_and_tracks_f64():
    """The fp32 instantiation of the Eq. 1 blend (Sec. 3.1): against the blend of two library
    attentions (float64 SDPA over the full and the local position set) and against its fp64 twin."""
    B, Hq, Hkv, cap, D, S, R = 2, 14, 2, 700, 128, 16, 64
    k, v, q = _rand(23, B, Hq, Hkv, cap, D, torch.bfloat16)
    n, gate, scale = [700, 333], [0.3, 0.85], 1 / math.sqrt(D)
    a = oracle.decode_attention_gated(_np(k), _np(v), n, gate, _np(q), S, R, scale)
    b_ = oracle.decode_attention_gated(_np(k), _np(v), n, gate, _np(q), S, R, scale, precision="f32")
    assert b_.dtype == np.float32
    assert np.abs(a - b_).max() < 2e-6
    G = Hq // Hkv
    for b in range(B):
        rows_local = [j for j in range(n[b]) if j < S or j >= n[b] - R]
        full = _sdpa_rows(k[b].float(), v[b].float(), q[b].float(), list(range(n[b])), scale, G)
        local = _sdpa_rows(k[b].float(), v[b].float(), q[b].float(), rows_local, scale, G)
        for i in range(Hq):
            g = gate[i // G]
            np.testing.assert_allclose(b_[b, i], g * full[i] + (1 - g) * local[i], rtol=0, atol=2e-6)
    # gate 1 / 0 reduce to the binary head kinds in the fp32 variant too
    o1 = oracle.decode_attention_gated(_np(k), _np(v), n, [1, 0], _np(q), S, R, scale, precision="f32")
    ob = oracle.decode_attention(_np(k), _np(v), n, [1, 0], _np(q), S, R, scale, precision="f32")
    np.testing.assert_allclose(o1, ob, rtol=0, atol=1e-6)


# ---------------------------------------------------------------- prefill with mask matrices

def _mask_matrices(n_old, t, S, R):
    """Rows n_old .. n_old + t - 1 of the causal and the local mask, written out as matrices
    over all keys 0 .. n_old + t - 1 (numpy, independent of the oracle's loops)."""
    i = np.arange(n_old, n_old + t)[:, None]
    j = np.arange(n_old + t)[None, :]
    causal = j <= i
    local = causal & ((j < S) | (i - j < R))
    return causal, local


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("S,R", [(4, 10), (0, 3), (16, 48)])
def test_prefill_equals_library_attention_under_mask_matrices(dtype, S, R):
    B, Hq, Hkv, cap, D, T = 3, 6, 3, 140, 32, 50
    k = synth.normal(31, synth.T_K, 0, range(B), range(Hkv), 0, cap, D, dtype=dtype)
    v = synth.normal(31, synth.T_V, 0, range(B), range(Hkv), 0, cap, D, dtype=dtype)
    q = synth.normal(31, synth.T_Q, 0, range(B), range(Hq), 0, T, D, dtype=dtype)
    n_old, t = [0, 90, 77], [50, 37, 0]
    gate = [1.0, 0.0, 0.4]
    scale, G = 0.3, Hq // Hkv
    out = oracle.prefill_attention(_np(k), _np(v), n_old, t, gate, _np(q), S, R, scale)
    for b in range(B):
        assert np.isnan(out[b, :, t[b]:]).all()            # rows past the chunk are not produced
        if t[b] == 0:
            continue
        n = n_old[b] + t[b]
        causal, local = _mask_matrices(n_old[b], t[b], S, R)
        kk = k[b].double()[:, :n].repeat_interleave(G, dim=0)[None]
        vv = v[b].double()[:, :n].repeat_interleave(G, dim=0)[None]
        qq = q[b].double()[:, :t[b]][None]
        sdpa = torch.nn.functional.scaled_dot_product_attention
        o_c = sdpa(qq, kk, vv, attn_mask=torch.from_numpy(causal), scale=scale)[0].numpy()
        o_l = sdpa(qq, kk, vv, attn_mask=torch.from_numpy(local), scale=scale)[0].numpy()
        for hq in range(Hq):
            a = gate[hq // G]
            np.testing.assert_allclose(out[b, hq, :t[b]], a * o_c[hq] + (1 - a) * o_l[hq], rtol=0, atol=1e-12)


def test_prefill_rows_equal_decode_steps():
    """Row c of a prefill chunk is the decode step that sees n_old + c + 1 cached positions."""
    B, Hq, Hkv, cap, D, T, S, R = 2, 4, 2, 60, 16, 20, 3, 6
    k = synth.normal(32, synth.T_K, 0, range(B), range(Hkv), 0, cap, D, dtype=torch.float32)
    v = synth.normal(32, synth.T_V, 0, range(B), range(Hkv), 0, cap, D, dtype=torch.float32)
    q = synth.normal(32, synth.T_Q, 0, range(B), range(Hq), 0, T, D, dtype=torch.float32)
    n_old, t = [0, 40], [20, 11]
    gate = [1.0, 0.0]
    out = oracle.prefill_attention(_np(k), _np(v), n_old, t, gate, _np(q), S, R, 0.25)
    for c in range(T):
        live = [b for b in range(B) if c < t[b]]
        if not live:
            continue
        n = [n_old[b] + c + 1 for b in range(B)]
        step = oracle.decode_attention(_np(k), _np(v), n, [1, 0], np.ascontiguousarray(_np(q)[:, :, c]), S, R, 0.25)
        for b in live:
            np.testing.assert_allclose(out[b, :, c], step[b], rtol=0, atol=1e-14)


def test_prefill_zero_keys_give_the_mean_of_the_mask_row():
    """K = 0 -> uniform weights; with V[j][d] = j the output is the mean of the admitted positions:
    (i + 1 - 1) / 2 = i / 2 under the causal mask; (sum of sinks + sum of the last R) / (S + R) under
    the local mask once i + 1 > S + R."""
    B, Hq, Hkv, cap, D, T, S, R = 1, 2, 2, 64, 8, 24, 3, 5
    k = np.zeros((B, Hkv, cap, D), dtype=np.float32)
    v = np.broadcast_to(np.arange(cap, dtype=np.float32)[None, None, :, None], (B, Hkv, cap, D)).copy()
    q = np.ones((B, Hq, T, D), dtype=np.float32)
    n_old = 30
    out = oracle.prefill_attention(k, v, [n_old], [T], [1.0, 0.0], q, S, R, 1.0)
    for c in range(T):
        i = n_old + c
        np.testing.assert_allclose(out[0, 0, c], i / 2.0, atol=1e-12)
        expect = (sum(range(S)) + sum(range(i - R + 1, i + 1))) / (S + R)
        np.testing.assert_allclose(out[0, 1, c], expect, atol=1e-12)


def test_prefill_f32_variant_is_pinned_to_mask_matrices_and_tracks_f64():
    """The fp32 instantiation of prefill (Sec. 3.1 masks, App. B): against library attention under
    explicit mask matrices (float64 SDPA) and against its fp64 twin, rows past a chunk left NaN."""
    B, Hq, Hkv, cap, D, T, S, R = 2, 6, 3, 400, 128, 70, 8, 40
    k = synth.normal(33, synth.T_K, 0, range(B), range(Hkv), 0, cap, D, dtype=torch.bfloat16)
    v = synth.normal(33, synth.T_V, 0, range(B), range(Hkv), 0, cap, D, dtype=torch.bfloat16)
    q = synth.normal(33, synth.T_Q, 0, range(B), range(Hq), 0, T, D, dtype=torch.bfloat16)
    n_old, t, gate = [330, 0], [70, 41], [1.0, 0.0, 0.6]
    scale, G = 1 / math.sqrt(D), Hq // Hkv
    a = oracle.prefill_attention(_np(k), _np(v), n_old, t, gate, _np(q), S, R, scale)
    b_ = oracle.prefill_attention(_np(k), _np(v), n_old, t, gate, _np(q), S, R, scale, precision="f32")
    assert b_.dtype == np.float32
    sdpa = torch.nn.functional.scaled_dot_product_attention
    for b in range(B):
        assert np.isnan(b_[b, :, t[b]:]).all()
        assert np.abs(a[b, :, :t[b]] - b_[b, :, :t[b]]).max() < 2e-6
        n = n_old[b] + t[b]
        causal, local = _mask_matrices(n_old[b], t[b], S, R)
        kk = k[b].double()[:, :n].repeat_interleave(G, dim=0)[None]
        vv = v[b].double()[:, :n].repeat_interleave(G, dim=0)[None]
        qq = q[b].double()[:, :t[b]][None]
        o_c = sdpa(qq, kk, vv, attn_mask=torch.from_numpy(causal), scale=scale)[0].numpy()
        o_l = sdpa(qq, kk, vv, attn_mask=torch.from_numpy(local), scale=scale)[0].numpy()
        for hq in range(Hq):
            g = gate[hq // G]
            np.testing.assert_allclose(b_[b, hq, :t[b]], g * o_c[hq] + (1 - g) * o_l[hq], rtol=0, atol=2e-6)


def test_prefill_invalid_arguments():
    k = np.zeros((1, 1, 8, 4), dtype=np.float32)
    q = np.zeros((1, 1, 4, 4), dtype=np.float32)
    for bad in (dict(n_old=[6], t=[3]), dict(n_old=[0], t=[5]), dict(n_old=[-1], t=[1])):
        with pytest.raises(ValueError):
            oracle.prefill_attention(k, k, bad["n_old"], bad["t"], [1.0], q, 1, 1, 1.0)
    with pytest.raises(ValueError):
        oracle.prefill_attention(k, k, [0], [2], [1.2], q, 1, 1, 1.0)


# ---------------------------------------------------------------- ring-buffer indices

def _closed_form_slots(S, R, n):
    out = np.full(S + R, -1, dtype=np.int32)
    for t in range(S):
        if t < n:
            out[t] = t
    for r in range(R):
        # largest p < n with p >= S and (p - S) % R == r
        if n - 1 - S >= r:
            out[S + r] = S + r + R * ((n - 1 - S - r) // R)
    return out


@pytest.mark.parametrize("S,R", [(16, 112), (0, 4), (4, 1), (64, 256), (3, 7)])
def test_ring_simulation_matches_closed_form_and_position_set(S, R):
    W = S + R
    for n in [0, 1, S, S + 1, W - 1, W, W + 1, W + R, 2 * R + S + 3, 5 * W + 11]:
        slots, length = oracle.ring_simulate(S, R, n)
        assert length == n
        np.testing.assert_array_equal(slots, _closed_form_slots(S, R, n))
        held = sorted(int(p) for p in slots if p >= 0)
        expect = [j for j in range(n) if j < S or j >= n - R]
        assert held == expect                       # the store holds exactly the position set
        assert len(held) == min(n, W)               # constant size once full
        # filled slots form a prefix of the store
        assert all(slots[i] >= 0 for i in range(min(n, W))) and all(slots[i] < 0 for i in range(min(n, W), W))


# ---------------------------------------------------------------- bytes model

def test_bytes_model_reproduces_printed_theoretical_speedups():
    """KV bytes all-full / mixed == 1/((1-s)+sW/L); the paper prints it for W=80."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table3_theoretical.txt")) if l.strip() and l[0] != "#"]
    W_s, W_r, L = 16, 64, 2880
    for s_txt, printed in rows:
        s = float(s_txt)
        hkv = 10
        w = workloads.Workload("t", 1, hkv, hkv, 128, "bf16", 1, L, L, 0, W_s, W_r, 1, 0)
        mask = np.ones((1, hkv), dtype=np.uint8)
        mask[0, :int(round(s * hkv))] = 0
        kv_only = lambda m: workloads.algorithmic_bytes_per_step(w, [L], m) - 1 * 1 * (2 * hkv * 128 * 2 + 2 * hkv * 128 * 2)
        ratio = kv_only(np.ones_like(mask)) / kv_only(mask)
        closed = 1.0 / ((1 - s) + s * (W_s + W_r) / L)
        assert abs(ratio - closed) < 1e-12
        assert f"{closed:.2f}" == printed


# ---------------------------------------------------------------- generator sanity

def test_generator_is_deterministic_and_slice_consistent():
    a = synth.normal(7, synth.T_K, 3, [0, 5], [1, 2], 0, 64, 128, dtype=torch.bfloat16)
    b = synth.normal(7, synth.T_K, 3, [5], [2], 16, 8, 128, dtype=torch.bfloat16)
    assert torch.equal(a[1:2, 1:2, 16:24], b)
    c = synth.normal(7, synth.T_K, 3, [0], [1], 0, 8, 128, sink_scale=4.0, n_sink_scaled=4)
    d = synth.normal(7, synth.T_K, 3, [0], [1], 0, 8, 128)
    assert torch.equal(c[:, :, :4], 4 * d[:, :, :4]) and torch.equal(c[:, :, 4:], d[:, :, 4:])
    x = synth.normal(7, synth.T_V, 0, range(4), range(4), 0, 512, 128)
    assert abs(float(x.mean())) < 5e-3 and abs(float(x.std()) - 1) < 5e-3


def test_head_mask_counts():
    for name, total in [("c2", 51), ("c3", 67), ("c4", 153), ("c5", 153)]:
        w = workloads.WORKLOADS[name]
        m = w.mask()
        assert m.shape == (w.n_layers, w.n_kv_heads)
        assert int((m == 0).sum()) == total
        per_layer = (m == 0).sum(1)
        assert per_layer.max() - per_layer.min() <= 1
    m1 = workloads.WORKLOADS["c1"].mask()
    assert m1.tolist() == [[1, 1, 1, 1, 0, 0, 0, 0]]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_split_merge_of_partials_equals_the_unsplit_result(seed):
    """The merge step of split-K attention: cut the position set into arbitrary parts, form each part's
    (m, l, acc) = (max score, sum of exp(s - m), sum of exp(s - m) v), and merge with
    M = max m_i, out = sum e^(m_i - M) acc_i / sum e^(m_i - M) l_i.  For any partition this is the
    oracle's unsplit output (empty parts, with m = -inf, drop out).  Written here with numpy only."""
    rng = np.random.RandomState(seed)
    S, R = 4, 9
    B, Hq, Hkv, cap, D = 1, 6, 2, 80, 16
    k, v, q = _rand(30 + seed, B, Hq, Hkv, cap, D)
    n, scale = [cap - seed], 0.7
    ref = oracle.decode_attention(_np(k), _np(v), n, [1, 0], _np(q), S, R, scale)
    kd, vd, qd = k.double().numpy(), v.double().numpy(), q.double().numpy()
    for i in range(Hq):
        h = i // (Hq // Hkv)
        pos = [j for j in range(n[0]) if oracle.in_position_set(h == 0, j, n[0], S, R)]
        order = rng.permutation(pos)
        cuts = sorted(rng.choice(len(order) + 1, size=5))          # may repeat: empty parts
        parts = np.split(order, cuts)
        ms, ls, accs = [], [], []
        for part in parts:
            if len(part) == 0:
                ms.append(-np.inf); ls.append(0.0); accs.append(np.zeros(D))
                continue
            s = scale * kd[0, h, part] @ qd[0, i]
            m = s.max()
            w = np.exp(s - m)
            ms.append(m); ls.append(w.sum()); accs.append(w @ vd[0, h, part])
        M = max(ms)
        f = [0.0 if m == -np.inf else np.exp(m - M) for m in ms]
        out = sum(fi * a for fi, a in zip(f, accs)) / sum(fi * l for fi, l in zip(f, ls))
        np.testing.assert_allclose(out, ref[0, i], rtol=1e-12, atol=1e-13)
