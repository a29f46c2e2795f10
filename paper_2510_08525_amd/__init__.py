"""MI355X-native decode attention over a head-mixed KV cache (RLKV hot path).

The product is the C-ABI library `librlkv.so` (hand-written HIP for gfx950, see
include/rlkv.h).  This package is the thin Python binding over it: argument marshalling
only; PyTorch provides device memory and streams.
"""
from .binding import (RLKV_BF16, RLKV_F32, RLKV_KERNEL_AUTO, RLKV_KERNEL_MFMA,  # noqa: F401
                      RLKV_KERNEL_VALU, Cache, RlkvError, library_path, load_library,
                      rlkv_append, rlkv_append_decode, rlkv_append_decode_launch, rlkv_append_decode_prepare, rlkv_append_ragged, rlkv_cache_create, rlkv_cache_destroy,
                      rlkv_cache_kernel, rlkv_cache_required_bytes, rlkv_cache_reset,
                      rlkv_decode_attention, rlkv_decode_attention_noalloc, rlkv_get_lengths, rlkv_get_slot_positions, rlkv_profile_collect, rlkv_profile_enable,
                      rlkv_pool_pages_free, rlkv_pool_shuffle, rlkv_plan_prefill_form, rlkv_plan_prefill_block, rlkv_plan_prefill_rows, rlkv_plan_shares, rlkv_prefill_attention, rlkv_probe_stream_read, rlkv_resident_bytes, rlkv_set_active, rlkv_set_gates, rlkv_status_string, rlkv_worklists_built)
