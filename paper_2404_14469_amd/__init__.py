"""MI355X-native SnapKV prompt-KV compression (arXiv 2404.14469, Sec. 4.1 / Listing 1).

The product is libsnapkv.so (HIP kernels for gfx950 behind the C ABI of include/snapkv.h);
this package is its thin Python binding plus the seeded synthetic workload generator.
"""
from .binding import (DTYPE_BF16, DTYPE_F16, DTYPE_F32, LIB_PATH, ERR_TIMEOUT, POOL_AVG, POOL_MAX, STATIC_SCRATCH_BYTES, SYMBOLS, SnapKVError,
                      compress, load, snapkv_compress, snapkv_compress_lse, snapkv_capacity_for_rate, snapkv_compress_paged, snapkv_compress_per_query_head, snapkv_compress_strided, snapkv_compress_varlen, snapkv_compress_layers, snapkv_compress_static, snapkv_compress_ws_status, snapkv_debug_set_wait_limit, snapkv_decode_attention, snapkv_hit_rate, snapkv_pooled_scores,
                      snapkv_pooled_scores_lse, snapkv_profile_start,
                      snapkv_profile_stop, snapkv_release, snapkv_set_scoring_scheme, snapkv_sync_timeouts,
                      snapkv_select_topk, snapkv_strerror, snapkv_version, snapkv_workspace_bytes)

__all__ = ["DTYPE_BF16", "DTYPE_F16", "DTYPE_F32", "LIB_PATH", "ERR_TIMEOUT", "POOL_AVG", "POOL_MAX", "STATIC_SCRATCH_BYTES", "SYMBOLS", "SnapKVError",
           "compress", "load", "snapkv_compress", "snapkv_compress_lse", "snapkv_capacity_for_rate", "snapkv_compress_paged", "snapkv_compress_per_query_head", "snapkv_compress_strided", "snapkv_compress_varlen", "snapkv_compress_layers", "snapkv_compress_static", "snapkv_compress_ws_status", "snapkv_debug_set_wait_limit", "snapkv_decode_attention", "snapkv_hit_rate", "snapkv_pooled_scores",
           "snapkv_pooled_scores_lse", "snapkv_profile_start", "snapkv_profile_stop", "snapkv_release", "snapkv_set_scoring_scheme", "snapkv_sync_timeouts",
           "snapkv_select_topk", "snapkv_strerror", "snapkv_version", "snapkv_workspace_bytes"]
