"""Shared driver for the GPU parity tests: runs the HIP path and the oracle on the same
seeded inputs and compares them element by element."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2510_08525_amd as rl
from inputs import synth

# fp32 config: scores and sums in fp32 on both sides (oracle in fp64): a few 1e-6 of
# rounding on O(1) outputs.
# bf16: the bar is 1e-2 absolute (unit-scale outputs).  The output is rounded to bf16, so an
# error of half a bf16 ulp at the reference is unavoidable: 2^(e-8) for |ref| in [2^e, 2^(e+1)),
# which exceeds 1e-2 only from |ref| >= 4 on.  There the tolerance is that half ulp plus
# ACC_EPS * |ref| for the error before the final rounding (fp32 accumulation; weights carried
# with >= 11 significant bits, whose common truncation cancels against the normaliser), which can
# push a value across a rounding boundary.  Below |ref| = 4 the flat bar applies unrelaxed.
TOL_F32 = 1e-5
TOL_BF16 = 1e-2
ACC_EPS = 2.0 ** -11


def bf16_half_ulp(ref: np.ndarray) -> np.ndarray:
    """Half the spacing of bf16 values (8 significant bits) at |ref|."""
    _, ex = np.frexp(np.abs(ref))              # |ref| = m * 2^ex, m in [0.5, 1)
    return np.ldexp(1.0, ex - 9)


def tolerance(ref: np.ndarray, dtype: int, rel: float = 0.0) -> np.ndarray:
    """The one definition of the parity tolerance (tests and the benchmark's spot checks).
    rel: extra relative allowance for tests whose V is far from unit scale."""
    ref = np.asarray(ref, dtype=np.float64)
    if dtype == rl.RLKV_F32:
        return np.full_like(ref, TOL_F32)
    return np.maximum(TOL_BF16, bf16_half_ulp(ref) + ACC_EPS * np.abs(ref)) + rel * np.abs(ref)


def to_np(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu()
    return synth.bf16_bits(t) if t.dtype == torch.bfloat16 else t.numpy()


def expected_slot_positions(sink: int, recent: int, n: int) -> np.ndarray:
    return oracle.ring_simulate(sink, recent, n)[0]


# rlkv_config_t tuning fields every Case creates its cache with (a fixture may set them for a test)
TUNING: dict = {}


class Case:
    """One single-layer-at-a-time scenario with a complete CPU-side K/V history."""

    def __init__(self, *, Hq, Hkv, B, S, R, dtype, kernel, mask, cap, seed=1, n_layers=1, layer=0,
                 scale=None, sink_keys=True, device="cuda:0", q_prescale=1.0, arena_fill=None, page_tokens=0,
                 pool_pages=0, prefill_tokens=0):
        self.Hq, self.Hkv, self.B, self.S, self.R = Hq, Hkv, B, S, R
        self.D = 128
        self.dtype, self.kernel = dtype, kernel
        self.tdtype = torch.float32 if dtype == rl.RLKV_F32 else torch.bfloat16
        self.layer, self.n_layers = layer, n_layers
        self.mask_layer = np.asarray(mask, dtype=np.uint8).reshape(Hkv)
        full_mask = np.ones((n_layers, Hkv), dtype=np.uint8)
        full_mask[layer] = self.mask_layer
        self.cap = cap
        self.scale = scale if scale is not None else 1.0 / np.sqrt(self.D)
        self.device = torch.device(device)
        self.seed = seed
        self.q_prescale = q_prescale
        # complete history on the CPU (what the oracle sees)
        kw = dict(sink_scale=4.0, n_sink_scaled=4) if sink_keys else {}
        self.k_hist = synth.normal(seed, synth.T_K, layer, range(B), range(Hkv), 0, cap, self.D,
                                   dtype=self.tdtype, **kw)
        self.v_hist = synth.normal(seed, synth.T_V, layer, range(B), range(Hkv), 0, cap, self.D, dtype=self.tdtype)
        self.n = np.zeros(B, dtype=np.int64)
        self.cache = rl.Cache(n_layers, Hq, Hkv, self.D, B, S, R, dtype, full_mask, [cap] * B,
                              kernel=kernel, device=device, arena_fill=arena_fill, page_tokens=page_tokens,
                              pool_pages=pool_pages, prefill_tokens=prefill_tokens, **TUNING)

    def close(self):
        self.cache.close()

    # -- HIP path --------------------------------------------------------------------
    def append(self, counts):
        """Append counts[b] tokens (the next rows of the history) to every sequence."""
        counts = np.asarray(counts, dtype=np.int64).reshape(self.B)
        stride = int(max(1, counts.max()))
        k = torch.zeros(self.B, self.Hkv, stride, self.D, dtype=self.tdtype)
        v = torch.zeros_like(k)
        for b in range(self.B):
            c = int(counts[b])
            k[b, :, :c] = self.k_hist[b, :, self.n[b]:self.n[b] + c]
            v[b, :, :c] = self.v_hist[b, :, self.n[b]:self.n[b] + c]
        kd, vd = k.to(self.device), v.to(self.device)
        if (counts == counts[0]).all() and counts[0] > 0:
            self.cache.append(self.layer, kd, vd)
        else:
            self.cache.append_ragged(self.layer, kd, vd, counts.astype(np.int32))
        self.n += counts

    def make_q(self, step_id):
        q = synth.normal(self.seed, synth.T_Q, self.layer, range(self.B), range(self.Hq), step_id, 1, self.D,
                         dtype=torch.float32)[:, :, 0, :]
        return (q * self.q_prescale).to(self.tdtype).contiguous()

    def append_decode(self, step_id=0):
        """One fused step: append the next history row of every sequence, then attend."""
        k = torch.stack([self.k_hist[b, :, self.n[b]:self.n[b] + 1] for b in range(self.B)]).contiguous()
        v = torch.stack([self.v_hist[b, :, self.n[b]:self.n[b] + 1] for b in range(self.B)]).contiguous()
        q = self.make_q(step_id)
        out = torch.full((self.B, self.Hq, self.D), float("nan"), dtype=self.tdtype, device=self.device)
        self.cache.append_decode(self.layer, k.to(self.device), v.to(self.device), q.to(self.device), out, self.scale)
        torch.cuda.synchronize()
        self.n += 1
        return q, out

    def decode(self, step_id=0):
        q = synth.normal(self.seed, synth.T_Q, self.layer, range(self.B), range(self.Hq), step_id, 1, self.D,
                         dtype=torch.float32)[:, :, 0, :]
        q = (q * self.q_prescale).to(self.tdtype).contiguous()
        qd = q.to(self.device)
        out = torch.full((self.B, self.Hq, self.D), float("nan"), dtype=self.tdtype, device=self.device)
        self.cache.decode_attention(self.layer, qd, out, self.scale)
        torch.cuda.synchronize()
        return q, out

    def check_prefill(self, counts, step_id=0, label="", stride=None, gates=None, rel=0.0):
        """One chunk through rlkv_prefill_attention (attention under the causal / local mask, then
        the append), compared row by row with the oracle's prefill on the complete history."""
        counts = np.asarray(counts, dtype=np.int64).reshape(self.B)
        stride = int(stride or max(1, counts.max()))
        k = torch.zeros(self.B, self.Hkv, stride, self.D, dtype=self.tdtype)
        v = torch.zeros_like(k)
        for b in range(self.B):
            c = int(counts[b])
            k[b, :, :c] = self.k_hist[b, :, self.n[b]:self.n[b] + c]
            v[b, :, :c] = self.v_hist[b, :, self.n[b]:self.n[b] + c]
        q = synth.normal(self.seed, synth.T_Q, self.layer, range(self.B), range(self.Hq), 100000 * (step_id + 1),
                         stride, self.D, dtype=torch.float32)
        q = (q * self.q_prescale).to(self.tdtype).contiguous()
        out = torch.full((self.B, self.Hq, stride, self.D), 7.0, dtype=self.tdtype, device=self.device)
        self.cache.prefill_attention(self.layer, q.to(self.device), k.to(self.device), v.to(self.device),
                                     counts.astype(np.int32), out, self.scale)
        torch.cuda.synchronize()
        self.last_out = out
        n_old = self.n.copy()
        self.n += counts
        # the oracle's gate per KV head: 1 = causal mask, 0 = local mask (a compressed head), between = Eq. 1 blend
        eff = [float(m) for m in self.mask_layer] if gates is None else \
              [float(g) if m else 0.0 for g, m in zip(gates, self.mask_layer)]
        ref = oracle.prefill_attention(to_np(self.k_hist), to_np(self.v_hist), n_old, counts, eff, to_np(q),
                                       self.S, self.R, self.scale)
        got = out.float().cpu().numpy().astype(np.float64)
        worst = 0.0
        for b in range(self.B):
            c = int(counts[b])
            assert (got[b, :, c:] == 7.0).all(), f"{label}: rows past the chunk of sequence {b} were written"
            if c == 0:
                continue
            g, r = got[b, :, :c], ref[b, :, :c]
            assert np.isfinite(g).all(), f"{label}: non-finite output in sequence {b}"
            err = np.abs(g - r)
            bad = err > tolerance(r, self.dtype, rel)
            assert not bad.any(), (f"{label}: seq {b} max err {err.max():.3e} at "
                                   f"{np.unravel_index(err.argmax(), err.shape)} (n_old={n_old.tolist()}, "
                                   f"counts={counts.tolist()}, {bad.sum()} elements over tolerance)")
            worst = max(worst, float(err.max()))
        return worst

    # -- checks ----------------------------------------------------------------------
    def check_indices(self):
        lens = self.cache.lengths(self.layer)
        np.testing.assert_array_equal(lens, self.n.astype(np.int32))
        for h in range(self.Hkv):
            if self.mask_layer[h]:
                continue
            for b in range(self.B):
                got = self.cache.slot_positions(self.layer, h, b)
                np.testing.assert_array_equal(got, expected_slot_positions(self.S, self.R, int(self.n[b])),
                                              err_msg=f"slot positions head {h} seq {b} n {self.n[b]}")

    def check_decode(self, step_id=0, label="", fused=False, gates=None, rel=0.0):
        """gates: per-KV-head Eq. 1 gates already set on the cache (full heads only); the oracle
        then blends full and local attention for those heads."""
        q, out = self.append_decode(step_id) if fused else self.decode(step_id)
        if gates is None:
            ref = oracle.decode_attention(to_np(self.k_hist), to_np(self.v_hist), self.n, self.mask_layer, to_np(q),
                                          self.S, self.R, self.scale)
        else:
            # a compressed head is the gate-0 case: it only holds (and attends over) its local cache
            eff = [float(g) if m else 0.0 for g, m in zip(gates, self.mask_layer)]
            ref = oracle.decode_attention_gated(to_np(self.k_hist), to_np(self.v_hist), self.n, eff, to_np(q),
                                                self.S, self.R, self.scale)
        self.last_out = out
        got = out.float().cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all(), f"{label}: non-finite output"
        err = np.abs(got - ref)
        tol = tolerance(ref, self.dtype, rel)
        bad = err > tol
        assert not bad.any(), (f"{label}: max err {err.max():.3e} at {np.unravel_index(err.argmax(), err.shape)} "
                               f"(n={self.n.tolist()}, {bad.sum()} elements over tolerance)")
        return float(err.max())
