"""Paged full heads (paper Sec. 4.3: a standard paged cache for the full heads beside the
fixed-size buffers of the compressed ones), through the C-ABI.  Paging changes where rows
live, not what is computed: outputs must match the oracle within the usual tolerance and
equal the contiguous layout bit for bit (same work list, same order of operations); the
free-page count must follow the tokens cached; an exhausted pool must refuse an append
without writing anything."""
import numpy as np
import pytest
import torch

import paper_2510_08525_amd as rl
from paper_2510_08525_amd import binding
from harness import Case

pytestmark = pytest.mark.gpu

MFMA, BF16 = rl.RLKV_KERNEL_MFMA, rl.RLKV_BF16


def pages(n, page):
    return -(-int(n) // page)


@pytest.mark.parametrize("page", [32, 128, 512])
@pytest.mark.parametrize("Hq,Hkv,mask", [(32, 8, [1, 0, 1, 1, 0, 0, 1, 0]), (28, 4, [1, 0, 0, 1]), (8, 1, [1])])
def test_paged_equals_contiguous_and_oracle(gpu_device, page, Hq, Hkv, mask):
    """Ragged prefill over several pages, then fused steps that cross page and tile boundaries."""
    B, S, R, cap = 3, 8, 40, 1400
    lens = [1100, 37, 513]
    kw = dict(Hq=Hq, Hkv=Hkv, B=B, S=S, R=R, dtype=BF16, kernel=MFMA, mask=mask, cap=cap, seed=11)
    pool = sum(pages(n + 70, page) for n in lens) + 2
    paged = Case(page_tokens=page, pool_pages=pool, **kw)
    paged.cache.pool_shuffle(5)
    flat = Case(**kw)
    for c in (paged, flat):
        c.append([600, 37, 500])
        c.append([500, 0, 13])
        c.check_indices()
    assert paged.cache.pool_pages_free() == pool - sum(pages(n, page) for n in lens)
    assert flat.cache.pool_pages_free() == -1
    for step in range(70):
        fused = step % 3 != 2
        if not fused:
            for c in (paged, flat):
                c.append([1] * B)
        paged.check_decode(step, f"paged step {step}", fused=fused)
        flat.check_decode(step, f"contiguous step {step}", fused=fused)
        assert torch.equal(paged.last_out.cpu().view(torch.int16), flat.last_out.cpu().view(torch.int16)), f"step {step}"
    paged.check_indices()
    assert paged.cache.pool_pages_free() == pool - sum(pages(n, page) for n in paged.n)
    assert paged.cache.resident_bytes() < flat.cache.resident_bytes()
    paged.close()
    flat.close()


def test_pool_exhaustion_refuses_without_writing(gpu_device):
    page, B = 64, 2
    c = Case(Hq=8, Hkv=2, B=B, S=4, R=20, dtype=BF16, kernel=MFMA, mask=[1, 0], cap=2000, seed=4,
             page_tokens=page, pool_pages=6)
    c.append([128, 160])                       # 2 + 3 pages
    assert c.cache.pool_pages_free() == 1
    c.check_decode(0, "before")
    k = torch.zeros(B, 2, 64, 128, dtype=torch.bfloat16, device=c.device)
    with pytest.raises(rl.RlkvError) as e:     # needs 1 + 1 pages, one is left
        c.cache.append(0, k, k)
    assert e.value.status == binding.RLKV_ERR_CAPACITY
    assert c.cache.pool_pages_free() == 1
    c.check_indices()
    c.check_decode(1, "after the refused append")
    # one page is enough for a ragged append that only sequence 0 grows in
    c.append([64, 0])
    assert c.cache.pool_pages_free() == 0
    c.check_decode(2, "after taking the last page")
    # no page is needed while a sequence stays inside its last page ...
    for step in range(32):
        c.append([0, 1])                      # sequence 1 has room in its page until 192 tokens
    assert c.cache.pool_pages_free() == 0
    c.check_decode(70, "page of sequence 1 filled")
    with pytest.raises(rl.RlkvError) as e:
        c.append_decode(71)                   # ... and the fused step is refused when one of them needs a new one
    assert e.value.status == binding.RLKV_ERR_CAPACITY
    c.check_indices()
    # a reset returns the pages at once
    c.cache.reset(0)
    c.n[0] = 0
    assert c.cache.pool_pages_free() == 3
    c.append([10, 0])
    c.check_decode(72, "after reset and refill", fused=True)
    c.check_indices()
    c.close()


def test_pages_change_owner_after_reset(gpu_device):
    """Sequence 1 grows into the pages sequence 0 gave back; sequence 0 restarts shorter."""
    page = 32
    c = Case(Hq=28, Hkv=4, B=3, S=4, R=30, dtype=BF16, kernel=MFMA, mask=[1, 1, 0, 1], cap=900, seed=9,
             page_tokens=page, pool_pages=40)
    c.append([400, 100, 33])
    c.check_decode(0, "first fill")
    c.cache.reset(0)
    c.n[0] = 0
    c.append([0, 500, 0])                      # takes pages that held sequence 0
    c.append([90, 0, 200])
    c.check_indices()
    c.check_decode(1, "after hand-over")
    for step in range(2, 40):
        c.check_decode(step, f"fused {step}", fused=True)
    assert c.cache.pool_pages_free() == 40 - sum(pages(n, page) for n in c.n)
    c.cache.reset(-1)
    assert c.cache.pool_pages_free() == 40
    c.n[:] = 0
    c.append([5, 64, 65])
    c.check_decode(41, "after full reset")
    c.close()


def test_paged_with_gates_and_active_set(gpu_device):
    page = 64
    c = Case(Hq=32, Hkv=8, B=4, S=16, R=48, dtype=BF16, kernel=MFMA, mask=[1, 0, 1, 1, 0, 1, 0, 1], cap=800, seed=13,
             page_tokens=page, pool_pages=4 * 13)
    c.cache.pool_shuffle(77)
    c.append([300, 635, 64, 129])
    gates = np.array([0.3, 1, 0.0, 1.0, 1, 0.75, 1, 0.5], dtype=np.float32)
    c.cache.set_gates(gates)
    for step in range(10):
        c.check_decode(step, f"gated {step}", fused=step % 2 == 0, gates=gates)
    c.cache.set_gates(None)
    c.cache.set_active(np.array([1, 0, 1, 1], dtype=np.uint8))
    free_before = c.cache.pool_pages_free()
    k = torch.zeros(4, 8, 1, 128, dtype=torch.bfloat16, device=c.device)
    out = torch.full((4, 32, 128), 5.0, dtype=torch.bfloat16, device=c.device)
    q = c.make_q(99).to(c.device)
    assert c.n.tolist() == [305, 640, 69, 134]
    c.cache.append_decode(0, k, k, q, out, c.scale)     # slot 1 sits on a page boundary but is inactive: no page taken
    torch.cuda.synchronize()
    assert (out[1].float() == 5.0).all() and (out[0].float() != 5.0).any()
    assert c.cache.pool_pages_free() == free_before
    c.close()
