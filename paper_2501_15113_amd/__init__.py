"""Task-KV hot path on AMD MI355X: Python binding of libtaskkv (C ABI).

Argument marshalling only -- every step runs in the library's HIP kernels.
There is no CPU fallback: loading fails loudly when the library is not built.
"""
from .binding import (LayerCfg, TaskKVError, CHUNK_TOKENS, F32, BF16, PACK_SELECTIVE, PACK_NO_CACHE,
                      PACK_COMPRESSED, library_path, load_library,
                      taskkv_create, taskkv_destroy, taskkv_strerror, taskkv_workspace_bytes,
                      taskkv_cache_tokens, taskkv_hetero_head_count, taskkv_middle_budget,
                      taskkv_separate, taskkv_compress, taskkv_decode_attn, taskkv_cache_export,
                      taskkv_last_async_error, taskkv_profile_enable, taskkv_profile_read, taskkv_set_screening, taskkv_set_stream_skew, taskkv_set_stats_engine,
                      taskkv_stack_rebase, taskkv_decode_attn_layers, taskkv_decode_attn_static, taskkv_layer_plan,
                      EXPORTED_SYMBOLS)

__all__ = [
    "LayerCfg", "TaskKVError", "CHUNK_TOKENS", "F32", "BF16", "PACK_SELECTIVE", "PACK_NO_CACHE",
    "PACK_COMPRESSED", "library_path", "load_library",
    "taskkv_create", "taskkv_destroy", "taskkv_strerror", "taskkv_workspace_bytes",
    "taskkv_cache_tokens", "taskkv_hetero_head_count", "taskkv_middle_budget", "taskkv_separate",
    "taskkv_compress", "taskkv_decode_attn", "taskkv_cache_export", "taskkv_last_async_error",
    "taskkv_profile_enable", "taskkv_profile_read", "taskkv_set_screening", "taskkv_set_stream_skew", "taskkv_set_stats_engine", "taskkv_stack_rebase", "taskkv_decode_attn_layers",
    "taskkv_decode_attn_static", "taskkv_layer_plan", "EXPORTED_SYMBOLS",
]
