"""MI355X-native FP8-KV decode attention: thin Python binding of the C-ABI library libpz.so.

Every step of the path runs in the HIP kernels behind the C ABI declared in include/pz.h; this
package only marshals arguments (torch tensors supply device memory and streams).  There is no
CPU fallback: if the library has not been built, importing `binding` functions raises.
"""
from .binding import (APPEND_FORM_TILE, APPEND_FORM_TOKEN, KV_BF16, NOALLOC_WORKSPACE_BYTES, KV_FP8, OUT_BF16, OUT_F32, PagePool, PagedCache, PzError, YarnParams, lib, lib_path,
                      pz_debug_set_launch_override, pz_decode_attn, pz_decode_attn_append, pz_decode_attn_noalloc, pz_decode_attn_n_splits, pz_decode_attn_splitk_reduce,
                      pz_decode_attn_workspace_bytes, pz_kv_amax_update, pz_kv_append_fp8,
                      pz_kv_scales_from_amax, pz_prefill_attn, pz_rope_kv_append_fp8, pz_rope_yarn_table, pz_status_string,
                      pz_window_pages)

__all__ = ["APPEND_FORM_TILE", "APPEND_FORM_TOKEN", "KV_BF16", "NOALLOC_WORKSPACE_BYTES", "KV_FP8", "OUT_BF16", "OUT_F32", "PagePool", "PagedCache", "YarnParams", "PzError", "lib", "lib_path",
           "pz_debug_set_launch_override", "pz_decode_attn", "pz_decode_attn_append", "pz_decode_attn_noalloc", "pz_decode_attn_n_splits", "pz_decode_attn_splitk_reduce",
           "pz_decode_attn_workspace_bytes", "pz_kv_amax_update", "pz_kv_append_fp8", "pz_kv_scales_from_amax",
           "pz_prefill_attn", "pz_rope_kv_append_fp8", "pz_rope_yarn_table", "pz_status_string", "pz_window_pages"]
