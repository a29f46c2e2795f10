"""The allocation-free decode entry point (rlkv_decode_attention_noalloc), through the C-ABI: its split-K
partials live in the library's static device buffer instead of the arena.  Checked against
rlkv_decode_attention (bit for bit: same kernels, same order of operations) and against the oracle, on two
calls in a row of which the second is the smaller one, so that whatever the first left in the shared buffer
would show."""
import numpy as np
import pytest
import torch

import paper_2510_08525_amd as rl
from paper_2510_08525_amd import binding
from harness import Case

pytestmark = pytest.mark.gpu

BF16, F32 = rl.RLKV_BF16, rl.RLKV_F32
MFMA, VALU = rl.RLKV_KERNEL_MFMA, rl.RLKV_KERNEL_VALU


def _both_ways(c: Case, step_id: int, label: str, gates=None):
    """One decode step through the existing entry point (checked against the oracle) and through the
    allocation-free one; returns whether the two outputs have the same bits."""
    c.check_decode(step_id, label + ": rlkv_decode_attention", gates=gates)
    ref = c.last_out
    q = c.make_q(step_id).to(c.device)
    out = torch.full_like(ref, float("nan"))
    c.cache.decode_attention_noalloc(c.layer, q, out, c.scale)
    torch.cuda.synchronize()
    view = torch.int32 if ref.dtype == torch.float32 else torch.int16
    assert torch.equal(out.view(view), ref.view(view)), f"{label}: outputs differ from rlkv_decode_attention"


@pytest.mark.parametrize("dtype,kernel", [(BF16, MFMA), (BF16, VALU), (F32, VALU)], ids=["bf16-mfma", "bf16-valu", "f32-valu"])
def test_two_calls_in_a_row_the_second_smaller(gpu_device, dtype, kernel):
    big = Case(Hq=28, Hkv=4, B=6, S=16, R=112, dtype=dtype, kernel=kernel, mask=[1, 0, 0, 1], cap=5200, seed=91)
    big.append([5000, 4100, 333, 2900, 77, 1500])          # every full pair is split over many workgroups
    small = Case(Hq=28, Hkv=4, B=2, S=16, R=112, dtype=dtype, kernel=kernel, mask=[0, 1, 0, 0], cap=900, seed=92)
    small.append([800, 45])
    _both_ways(big, 0, "large call")
    _both_ways(small, 0, "smaller call after it")
    # and interleaved once more, with steps in between that go through the arena's partials
    big.append([1] * 6)
    _both_ways(big, 1, "large call again")
    small.append([3, 3])
    _both_ways(small, 1, "smaller call again")
    big.close()
    small.close()


def test_a_layer_that_blends_uses_two_sets_of_rows(gpu_device):
    c = Case(Hq=14, Hkv=2, B=3, S=8, R=40, dtype=BF16, kernel=MFMA, mask=[1, 1], cap=3000, seed=93)
    c.append([2900, 1000, 60])
    g = np.array([0.3, 1.0], dtype=np.float32)
    c.cache.set_gates(g)
    _both_ways(c, 0, "gated layer", gates=g)
    c.close()


def test_calls_beyond_the_static_buffer_are_refused(gpu_device):
    """(workgroups + pairs) * group size rows are needed: 4200 pairs of group size 4 exceed the 16384 rows."""
    B, Hkv, Hq = 1050, 4, 16
    cache = rl.Cache(1, Hq, Hkv, 128, B, 4, 28, BF16, [1, 0, 0, 1], [64] * B)
    k = torch.randn(B, Hkv, 40, 128, device="cuda:0").to(torch.bfloat16)
    cache.append(0, k, k)
    q = torch.randn(B, Hq, 128, device="cuda:0").to(torch.bfloat16)
    out = torch.zeros_like(q)
    ref = torch.zeros_like(q)
    cache.decode_attention(0, q, ref, 0.1)                  # the arena variant takes the call
    with pytest.raises(rl.RlkvError) as e:
        cache.decode_attention_noalloc(0, q, out, 0.1)
    assert e.value.status == binding.RLKV_ERR_TOO_LARGE
    torch.cuda.synchronize()
    assert (out == 0).all() and torch.isfinite(ref.float()).all()
    cache.close()
