"""MI355X-native PrefixKV hot path: thin Python binding over the C-ABI library libprefixkv.so.

Every step (importance, sort + cumulative priority, the search for the retention ratio p,
compaction, decode attention) runs in hand-written HIP kernels; this package only marshals
arguments.  PyTorch is used for device memory and streams.  There is no CPU fallback: importing
the binding without the built library raises.
"""
from .binding import (  # noqa: F401
    PKV_BF16, PKV_F32, PrefixKVError, SelectResult, RankResult, CompactResult, lib_path, load,
    prefixkv_cache_tokens_upper_bound, prefixkv_calibration_copy, prefixkv_compact, prefixkv_decode_attn, prefixkv_decode_attn_evict, prefixkv_gini, prefixkv_importance, prefixkv_merge_feature, prefixkv_merge_position,
    prefixkv_offline_config, prefixkv_prefill_attn, prefixkv_rank, prefixkv_select, prefixkv_select_static, prefixkv_static_scratch_segments, prefixkv_status_string, prefixkv_version, prefixkv_workspace_bytes, select_workspace_bytes,
)
