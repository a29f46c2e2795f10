"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol
the header declares, validates arguments before touching HIP, and sizes the arena."""
import os
import re

import numpy as np
import pytest

import paper_2510_08525_amd as rl
from paper_2510_08525_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _cfg(**over):
    kw = dict(n_layers=2, n_q_heads=8, n_kv_heads=2, head_dim=128, batch=3, sink=4, recent=8,
              dtype=rl.RLKV_BF16, full_mask=[1, 0, 0, 1], max_len=[100, 64, 33])
    kw.update(over)
    return kw


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "rlkv.h")).read()
    declared = set(re.findall(r"\b(rlkv_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTED_SYMBOLS)
    lib = rl.load_library()
    for name in declared:
        assert hasattr(lib, name), name


def test_required_bytes_accounts_for_stores():
    need = rl.rlkv_cache_required_bytes(**_cfg())
    # K+V rows: full heads hold round32(max_len) rows per sequence, compressed heads round32(S+R)
    row = 128 * 2
    full_rows = 128 + 64 + 64
    comp_rows = 32 * 3
    kv = 2 * row * (2 * full_rows + 2 * comp_rows)
    assert need >= kv
    assert need < kv + (64 << 20)
    # compressed stores do not grow with max_len; full stores do
    more = rl.rlkv_cache_required_bytes(**_cfg(max_len=[1124, 64, 33]))
    assert more - need == 2 * row * 2 * 1024
    allc = rl.rlkv_cache_required_bytes(**_cfg(full_mask=[0, 0, 0, 0], max_len=[100000, 64, 33]))
    allc2 = rl.rlkv_cache_required_bytes(**_cfg(full_mask=[0, 0, 0, 0]))
    assert allc == allc2


def test_paged_config_validation_and_sizing():
    """Paged full heads: the pool, not max_len, sizes the full stores."""
    ok = _cfg(page_tokens=64, pool_pages=4)
    need = rl.rlkv_cache_required_bytes(**ok)
    assert need > 0
    # four more pages in each of the 2 full heads' pools: 64 rows of K and V, bf16
    more = rl.rlkv_cache_required_bytes(**_cfg(page_tokens=64, pool_pages=8))
    assert more - need == 2 * 4 * 64 * 128 * 2 * 2
    huge = rl.rlkv_cache_required_bytes(**_cfg(page_tokens=64, pool_pages=4, max_len=[1 << 20, 64, 33]))
    assert huge - need < (1 << 20)                # only the block table grows with max_len
    for bad in (dict(page_tokens=48, pool_pages=4), dict(page_tokens=16, pool_pages=4),
                dict(page_tokens=64, pool_pages=0), dict(page_tokens=1 << 17, pool_pages=4),
                dict(page_tokens=64, pool_pages=4, kernel=rl.RLKV_KERNEL_VALU),
                dict(page_tokens=64, pool_pages=4, dtype=rl.RLKV_F32)):
        assert rl.rlkv_cache_required_bytes(**_cfg(**bad)) == 0, bad
    lib = rl.load_library()
    assert lib.rlkv_pool_pages_free(None) == -1
    assert lib.rlkv_pool_shuffle(None, 1) == binding.RLKV_ERR_INVALID_ARG


@pytest.mark.parametrize("bad", [
    dict(n_layers=0), dict(n_q_heads=7), dict(n_kv_heads=0), dict(head_dim=64), dict(batch=0),
    dict(sink=-1), dict(recent=0), dict(dtype=5), dict(kernel=9), dict(device=-1),
    dict(full_mask=[1, 0, 2, 1]), dict(max_len=[100, 0, 33]), dict(n_q_heads=64, n_kv_heads=2),
    dict(dtype=rl.RLKV_F32, kernel=rl.RLKV_KERNEL_MFMA),
    dict(decode_wgs_per_cu=9), dict(decode_wgs_per_cu=-1), dict(prefill_min_share_tiles=-3),
    dict(prefill_two_group_only=2),
    # (sequence, KV head) pairs index one grid dimension of several launches: at most 65535
    dict(batch=8192, n_kv_heads=8, n_q_heads=8, full_mask=[1] * 16, max_len=[32] * 8192),
])
def test_invalid_configs_rejected_on_host(bad):
    assert rl.rlkv_cache_required_bytes(**_cfg(**bad)) == 0
    with pytest.raises(rl.RlkvError) as e:
        rl.rlkv_cache_create(**_cfg(**bad))
    assert e.value.status == binding.RLKV_ERR_INVALID_ARG


def test_tuning_fields_accept_their_documented_range():
    base = rl.rlkv_cache_required_bytes(**_cfg())
    for ok in (dict(decode_wgs_per_cu=8), dict(prefill_min_share_tiles=8), dict(prefill_two_group_only=1)):
        assert rl.rlkv_cache_required_bytes(**_cfg(**ok)) == base, ok
    # the largest pair count the launches take
    assert rl.rlkv_cache_required_bytes(**_cfg(batch=65535, n_kv_heads=1, n_q_heads=1, full_mask=[0, 0],
                                               max_len=[32] * 65535)) > 0


def test_null_pointers_rejected():
    lib = rl.load_library()
    assert lib.rlkv_cache_required_bytes(None) == 0
    assert lib.rlkv_cache_create(None, None) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_cache_destroy(None) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_append(None, 0, None, None, 1, None) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_append_ragged(None, 0, None, None, None, 1, None) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_decode_attention(None, 0, None, None, 1.0, None) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_decode_attention_noalloc(None, 0, None, None, 1.0, None) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_cache_reset(None, -1, None) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_get_lengths(None, 0, None) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_get_slot_positions(None, 0, 0, 0, None) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_append_decode(None, 0, None, None, None, None, 1.0, None) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_append_decode_prepare(None, 0, None) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_append_decode_launch(None, 0, None, None, None, None, 1.0, None) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_worklists_built(None) == -1
    assert lib.rlkv_set_active(None, None, None) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_set_gates(None, None, None) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_profile_enable(None, 4) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_profile_collect(None, None, None) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_resident_bytes(None) == 0
    assert lib.rlkv_cache_kernel(None) == -1
    assert lib.rlkv_prefill_attention(None, 0, None, None, None, None, 1, None, 1.0, None) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_probe_stream_read(None, 16384, None, 1, None) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_pool_pages_free(None) == -1
    assert lib.rlkv_pool_shuffle(None, 0) == binding.RLKV_ERR_INVALID_ARG
    assert lib.rlkv_plan_shares(None, 1, 1, None, None, None) == -1


def test_prefill_config_validation():
    assert rl.rlkv_cache_required_bytes(**_cfg(prefill_tokens=512)) > rl.rlkv_cache_required_bytes(**_cfg())
    # the staging buffer: 3 sequences x 2 KV heads x 16 tiles of 16 KiB; and the scratch for the shares of divided
    # workgroups: 1024 slots of 256 columns x (128 + 2) fp32
    grow = rl.rlkv_cache_required_bytes(**_cfg(prefill_tokens=512)) - rl.rlkv_cache_required_bytes(**_cfg())
    assert grow == 3 * 2 * 16 * 16384 + 1024 * 256 * 130 * 4
    assert rl.rlkv_cache_required_bytes(**_cfg(prefill_tokens=-1)) == 0
    assert rl.rlkv_cache_required_bytes(**_cfg(prefill_tokens=64, kernel=rl.RLKV_KERNEL_VALU)) == 0
    assert rl.rlkv_cache_required_bytes(**_cfg(prefill_tokens=64, dtype=rl.RLKV_F32)) == 0


def test_misaligned_or_small_arena_rejected_before_hip():
    need = rl.rlkv_cache_required_bytes(**_cfg())
    with pytest.raises(rl.RlkvError) as e:
        rl.rlkv_cache_create(arena_ptr=0x1001, arena_bytes=need, **_cfg())
    assert e.value.status == binding.RLKV_ERR_INVALID_ARG
    with pytest.raises(rl.RlkvError) as e:
        rl.rlkv_cache_create(arena_ptr=0x1000, arena_bytes=need - 1, **_cfg())
    assert e.value.status == binding.RLKV_ERR_OOM


def test_status_strings():
    for s in range(7):
        assert rl.rlkv_status_string(s)
    assert rl.rlkv_status_string(0) == "ok"


def test_create_without_gpu_reports_hip_error():
    import torch

    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(rl.RlkvError) as e:
        rl.rlkv_cache_create(**_cfg())
    assert e.value.status == binding.RLKV_ERR_HIP


def test_binding_struct_matches_the_header(tmp_path):
    """The ctypes image of rlkv_config_t has the size and field offsets a C compiler gives the
    header's struct (compiled here with gcc as plain C, which also checks that the header is C)."""
    import ctypes
    import subprocess

    fields = [name for name, _ in binding._Config._fields_]
    src = tmp_path / "layout.c"
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "rlkv.h"', 'int main(void) {',
             '  printf("%zu\\n", sizeof(rlkv_config_t));']
    lines += [f'  printf("%zu\\n", offsetof(rlkv_config_t, {f}));' for f in fields]
    lines += ['  return 0;', '}']
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-std=c11", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    got = [int(x) for x in subprocess.check_output([str(exe)]).split()]
    assert got[0] == ctypes.sizeof(binding._Config)
    assert got[1:] == [getattr(binding._Config, f).offset for f in fields]


def test_bf16_tolerance_is_the_flat_bar_below_four_and_half_ulp_based_above():
    """The parity tolerance (tests/harness.py): 1e-2 wherever a bf16 result can meet it; from |ref| >= 4
    on, half the bf16 spacing at the reference plus the stated accumulation allowance, never more."""
    import numpy as np

    import harness

    bf16 = 1
    ref = np.array([0.0, 1e-3, 0.9, 2.56, 3.999, -3.5])
    np.testing.assert_array_equal(harness.tolerance(ref, bf16), np.full(6, 1e-2))
    # spacing of bf16 (8 significant bits) at 4 is 2^-5, at 100 (in [64, 128)) 2^-1
    np.testing.assert_allclose(harness.tolerance(np.array([4.0, -100.0]), bf16),
                               [2.0 ** -6 + 4.0 * harness.ACC_EPS, 2.0 ** -2 + 100.0 * harness.ACC_EPS], rtol=1e-15)
    # independent of the formula: the largest rounding error of torch's own bf16 conversion sits under it
    import torch
    x = torch.linspace(4.0, 300.0, 200001, dtype=torch.float64)
    err = (x.to(torch.float32).to(torch.bfloat16).double() - x).abs().numpy()
    assert (err <= harness.bf16_half_ulp(x.numpy()) * (1 + 1e-6)).all()
    assert (harness.tolerance(np.array([1.0]), 0) == 1e-5).all()


def test_header_and_example_are_plain_c():
    """include/rlkv.h is C (no C++ in the signatures): the example that drives the library from C passes a C11
    compiler's front end, warnings as errors."""
    import subprocess

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c11", "-Wall", "-Werror", "-fsyntax-only", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"),
           "-I", os.path.join(root, "include"), os.path.join(root, "examples", "c_abi_decode.c")]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
