"""Mixed attention with gating adapters (paper Sec. 3.1, Eq. 1) through the C-ABI:
gate * full attention + (1 - gate) * local attention on full heads, against the oracle."""
import numpy as np
import pytest
import torch

import paper_2510_08525_amd as rl
from paper_2510_08525_amd import binding
from harness import Case

pytestmark = pytest.mark.gpu

VARIANTS = [(rl.RLKV_F32, rl.RLKV_KERNEL_VALU), (rl.RLKV_BF16, rl.RLKV_KERNEL_VALU), (rl.RLKV_BF16, rl.RLKV_KERNEL_MFMA)]
IDS = ["f32-valu", "bf16-valu", "bf16-mfma"]


@pytest.mark.parametrize("dtype,kernel", VARIANTS, ids=IDS)
@pytest.mark.parametrize("Hq,Hkv", [(8, 4), (28, 4)])
def test_gated_token_by_token(gpu_device, dtype, kernel, Hq, Hkv):
    """Lengths 1..60 with S=4, R=12: before, at and past the point where local != full."""
    mask = [1, 1, 0, 1]
    gates = [0.3, 1.0, 0.7, 0.0]          # head 2 is compressed: its entry is ignored
    c = Case(Hq=Hq, Hkv=Hkv, B=2, S=4, R=12, dtype=dtype, kernel=kernel, mask=mask, cap=80, seed=41)
    c.cache.set_gates(gates)
    c.append([1, 5])
    for step in range(55):
        c.check_decode(step, f"gated step {step}", fused=(step % 2 == 0), gates=gates)
        if step % 2 == 1:
            c.append([1, 1])
    c.check_indices()
    # back to binary heads: same cache, plain full attention again
    c.cache.set_gates(None)
    c.check_decode(99, "gates cleared")
    c.close()


@pytest.mark.parametrize("dtype,kernel", VARIANTS, ids=IDS)
def test_gated_long_context_split_over_workgroups(gpu_device, dtype, kernel):
    """Thousands of tokens: the sink tiles and the recent tiles of a pair fall into different
    workgroups' shares, the middle shares contribute empty local partials."""
    gates = [0.25, 0.9]
    c = Case(Hq=14, Hkv=2, B=3, S=64, R=256, dtype=dtype, kernel=kernel, mask=[1, 1], cap=6100, seed=43)
    c.cache.set_gates(gates)
    c.append([6001, 3333, 300])
    c.check_decode(0, "gated prefill", gates=gates)
    for step in range(4):
        c.check_decode(step + 1, f"gated fused {step}", fused=True, gates=gates)
    # recent window not aligned to tiles, S = 0
    c.close()
    c = Case(Hq=4, Hkv=1, B=2, S=0, R=37, dtype=dtype, kernel=kernel, mask=[1], cap=900, seed=44)
    c.cache.set_gates([0.5])
    c.append([777, 38])
    for step in range(3):
        c.check_decode(step, f"S=0 gated {step}", fused=True, gates=[0.5])
    c.close()


def test_gate_validation(gpu_device):
    cache = rl.Cache(2, 4, 2, 128, 1, 4, 4, rl.RLKV_BF16, [1, 0, 1, 1], [32])
    for bad in ([0.5, 0.5, 1.5, 0.0], [0.5, 0.5, -0.1, 0.0], [float("nan"), 0, 0, 0]):
        with pytest.raises(rl.RlkvError) as e:
            cache.set_gates(bad)
        assert e.value.status == binding.RLKV_ERR_INVALID_ARG
    with pytest.raises(ValueError):
        cache.set_gates([0.5])
    cache.set_gates([0.5, 0.5, 1.0, 0.0])
    cache.close()
