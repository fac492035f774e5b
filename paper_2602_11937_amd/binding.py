"""ctypes binding of libpz.so: same names as the C entry points, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

_PKG = os.path.dirname(os.path.abspath(__file__))
KV_FP8, KV_BF16 = 0, 1
OUT_F32, OUT_BF16 = 0, 1


class PzError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s" % (where, pz_status_string(status)))


class _CCache(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("num_pages", C.c_int32),
                ("page_size", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("dtype", C.c_int32)]


class YarnParams(C.Structure):
    """pz_yarn_params; the defaults are the parent model's public configuration with the paper's factor."""
    _fields_ = [("theta", C.c_float), ("factor", C.c_float), ("original_context", C.c_int32),
                ("beta_fast", C.c_float), ("beta_slow", C.c_float)]

    def __init__(self, theta=150000.0, factor=56.0, original_context=4096, beta_fast=32.0, beta_slow=1.0):
        super().__init__(theta, factor, original_context, beta_fast, beta_slow)


def lib_path() -> str:
    return os.path.join(_PKG, "libpz.so")


_lib = None


def lib():
    """Load libpz.so (built by paper_2602_11937_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError("libpz.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(there is no CPU fallback for the decode-attention path)")
        L = C.CDLL(path)
        L.pz_status_string.restype = C.c_char_p
        L.pz_status_string.argtypes = [C.c_int]
        L.pz_debug_set_launch_override.restype = C.c_int
        L.pz_debug_set_launch_override.argtypes = [C.c_int32, C.c_int32]
        L.pz_kv_append_fp8.restype = C.c_int
        L.pz_kv_append_fp8.argtypes = [C.POINTER(_CCache), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                       C.c_float, C.c_float, C.c_void_p]
        L.pz_decode_attn_n_splits.restype = C.c_int32
        L.pz_decode_attn_n_splits.argtypes = [C.c_int32, C.c_int32, C.c_int32]
        L.pz_decode_attn_workspace_bytes.restype = C.c_size_t
        L.pz_decode_attn_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32]
        L.pz_decode_attn.restype = C.c_int
        L.pz_decode_attn.argtypes = [C.POINTER(_CCache), C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                     C.c_int32, C.c_int32, C.c_void_p, C.c_float, C.c_float, C.c_float,
                                     C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p,
                                     C.c_int32, C.c_void_p]
        L.pz_decode_attn_append.restype = C.c_int
        L.pz_decode_attn_append.argtypes = [C.POINTER(_CCache), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_float,
                                            C.c_float, C.c_float, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                            C.c_size_t, C.c_void_p, C.c_int32, C.c_void_p]
        L.pz_decode_attn_noalloc.restype = C.c_int
        L.pz_decode_attn_noalloc.argtypes = [C.POINTER(_CCache), C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                             C.c_int32, C.c_int32, C.c_void_p, C.c_float, C.c_float, C.c_float,
                                             C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p]
        L.pz_decode_attn_splitk_reduce.restype = C.c_int
        L.pz_decode_attn_splitk_reduce.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.c_int32, C.c_int32,
                                                   C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                                   C.c_float, C.c_void_p, C.c_int32, C.c_void_p]
        L.pz_kv_amax_update.restype = C.c_int
        L.pz_kv_amax_update.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        L.pz_kv_scales_from_amax.restype = C.c_int
        L.pz_kv_scales_from_amax.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        L.pz_prefill_attn.restype = C.c_int
        L.pz_prefill_attn.argtypes = [C.POINTER(_CCache), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                      C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_float, C.c_float, C.c_float,
                                      C.c_int32, C.c_void_p, C.c_int32, C.c_void_p]
        L.pz_rope_yarn_table.restype = C.c_int
        L.pz_rope_yarn_table.argtypes = [C.POINTER(YarnParams), C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.pz_rope_kv_append_fp8.restype = C.c_int
        L.pz_rope_kv_append_fp8.argtypes = [C.POINTER(_CCache), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32,
                                            C.c_float, C.c_float, C.c_void_p]
        L.pz_window_pages.restype = C.c_int32
        L.pz_window_pages.argtypes = [C.c_int32, C.c_int32]
        L.pz_page_pool_create.restype = C.c_void_p
        L.pz_page_pool_create.argtypes = [C.c_int32] * 5
        L.pz_page_pool_destroy.restype = None
        L.pz_page_pool_destroy.argtypes = [C.c_void_p]
        L.pz_page_pool_append.restype = C.c_int64
        L.pz_page_pool_append.argtypes = [C.c_void_p, C.c_int32]
        L.pz_page_pool_release.restype = C.c_int
        L.pz_page_pool_release.argtypes = [C.c_void_p, C.c_int32]
        L.pz_page_pool_seq_len.restype = C.c_int32
        L.pz_page_pool_seq_len.argtypes = [C.c_void_p, C.c_int32]
        L.pz_page_pool_free_pages.restype = C.c_int32
        L.pz_page_pool_free_pages.argtypes = [C.c_void_p]
        L.pz_page_pool_block_table.restype = C.POINTER(C.c_int32)
        L.pz_page_pool_block_table.argtypes = [C.c_void_p]
        L.pz_page_pool_drain_updates.restype = C.c_int32
        L.pz_page_pool_drain_updates.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32]
        L.pz_page_pool_pending_updates.restype = C.c_int32
        L.pz_page_pool_pending_updates.argtypes = [C.c_void_p]
        _lib = L
    return _lib


def pz_status_string(status: int) -> str:
    return lib().pz_status_string(int(status)).decode()


OVERRIDES = {"attn_waves": 0, "attn_chunks_per_group": 1, "attn_balanced": 2, "append_form": 3, "append_fused": 4}
APPEND_FORM_TILE, APPEND_FORM_TOKEN = 0, 1


def pz_debug_set_launch_override(which, value, check=True) -> int:
    """Force one launch-shape choice (tests and measurements); a negative value hands it back to the library.
    `which` is a pz_launch_override number or its lower-case name without the prefix."""
    st = lib().pz_debug_set_launch_override(int(OVERRIDES.get(which, which)), int(value))
    if check and st != 0:
        raise PzError(st, "pz_debug_set_launch_override")
    return st


def _ptr(t) -> Optional[int]:
    """Device (or raw) address of a torch tensor / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


@dataclass
class PagedCache:
    """Device K/V cache in the library's layout (K: [page][head][P][d], V: [page][head][d][P])."""
    k: object
    v: object
    num_pages: int
    page_size: int
    n_kv_heads: int
    head_dim: int
    dtype: int = KV_FP8

    @staticmethod
    def allocate(num_pages, page_size, n_kv_heads, head_dim, dtype=KV_FP8, device="cuda", fill=None):
        import torch
        tdt = torch.uint8 if dtype == KV_FP8 else torch.int16
        k = torch.empty((num_pages, n_kv_heads, page_size, head_dim), dtype=tdt, device=device)
        v = torch.empty((num_pages, n_kv_heads, head_dim, page_size), dtype=tdt, device=device)
        if fill is not None:
            k.fill_(fill)
            v.fill_(fill)
        return PagedCache(k, v, num_pages, page_size, n_kv_heads, head_dim, dtype)

    def c_struct(self) -> _CCache:
        return _CCache(_ptr(self.k), _ptr(self.v), self.num_pages, self.page_size, self.n_kv_heads,
                       self.head_dim, self.dtype)


def _cache_ref(cache):
    if cache is None:
        return None
    return C.byref(cache.c_struct() if isinstance(cache, PagedCache) else cache)


def pz_kv_append_fp8(cache, k_new, v_new, slot_mapping, n_tokens, k_scale, v_scale, stream=None,
                     check=True) -> int:
    st = lib().pz_kv_append_fp8(_cache_ref(cache), _ptr(k_new), _ptr(v_new), _ptr(slot_mapping),
                                int(n_tokens), float(k_scale), float(v_scale), _stream(stream))
    if check and st != 0:
        raise PzError(st, "pz_kv_append_fp8")
    return st


def pz_decode_attn_n_splits(max_seq_len, window, split_tokens) -> int:
    return int(lib().pz_decode_attn_n_splits(int(max_seq_len), int(window), int(split_tokens)))


def pz_decode_attn_workspace_bytes(batch, n_q_heads, head_dim, n_splits) -> int:
    return int(lib().pz_decode_attn_workspace_bytes(int(batch), int(n_q_heads), int(head_dim), int(n_splits)))


def pz_decode_attn(cache, q, block_table, max_pages_per_seq, seq_lens, batch, n_q_heads, sinks, sm_scale,
                   k_scale, v_scale, window, split_tokens, n_splits, workspace, workspace_bytes, out,
                   out_dtype=OUT_F32, stream=None, check=True) -> int:
    st = lib().pz_decode_attn(_cache_ref(cache), _ptr(q), _ptr(block_table), int(max_pages_per_seq),
                              _ptr(seq_lens), int(batch), int(n_q_heads), _ptr(sinks), float(sm_scale),
                              float(k_scale), float(v_scale), int(window), int(split_tokens), int(n_splits),
                              _ptr(workspace), int(workspace_bytes), _ptr(out), int(out_dtype),
                              _stream(stream))
    if check and st != 0:
        raise PzError(st, "pz_decode_attn")
    return st


NOALLOC_WORKSPACE_BYTES = 32 << 20


def pz_decode_attn_noalloc(cache, q, block_table, max_pages_per_seq, seq_lens, batch, n_q_heads, sinks, sm_scale,
                           k_scale, v_scale, window, split_tokens, n_splits, out, out_dtype=OUT_F32, stream=None,
                           check=True) -> int:
    st = lib().pz_decode_attn_noalloc(_cache_ref(cache), _ptr(q), _ptr(block_table), int(max_pages_per_seq),
                                      _ptr(seq_lens), int(batch), int(n_q_heads), _ptr(sinks), float(sm_scale),
                                      float(k_scale), float(v_scale), int(window), int(split_tokens), int(n_splits),
                                      _ptr(out), int(out_dtype), _stream(stream))
    if check and st != 0:
        raise PzError(st, "pz_decode_attn_noalloc")
    return st


def pz_decode_attn_append(cache, k_new, v_new, q, block_table, max_pages_per_seq, seq_lens, batch, n_q_heads, sinks,
                          sm_scale, k_scale, v_scale, window, split_tokens, n_splits, workspace, workspace_bytes, out,
                          out_dtype=OUT_F32, stream=None, check=True) -> int:
    st = lib().pz_decode_attn_append(_cache_ref(cache), _ptr(k_new), _ptr(v_new), _ptr(q), _ptr(block_table),
                                     int(max_pages_per_seq), _ptr(seq_lens), int(batch), int(n_q_heads), _ptr(sinks),
                                     float(sm_scale), float(k_scale), float(v_scale), int(window), int(split_tokens),
                                     int(n_splits), _ptr(workspace), int(workspace_bytes), _ptr(out), int(out_dtype),
                                     _stream(stream))
    if check and st != 0:
        raise PzError(st, "pz_decode_attn_append")
    return st


def pz_decode_attn_splitk_reduce(workspace, workspace_bytes, batch, n_q_heads, head_dim, n_splits, seq_lens,
                                 window, split_tokens, sinks, v_scale, out, out_dtype=OUT_F32, stream=None,
                                 check=True) -> int:
    st = lib().pz_decode_attn_splitk_reduce(_ptr(workspace), int(workspace_bytes), int(batch), int(n_q_heads),
                                            int(head_dim), int(n_splits), _ptr(seq_lens), int(window),
                                            int(split_tokens), _ptr(sinks), float(v_scale), _ptr(out),
                                            int(out_dtype), _stream(stream))
    if check and st != 0:
        raise PzError(st, "pz_decode_attn_splitk_reduce")
    return st


def pz_kv_amax_update(k, v, n_elems, amax, stream=None, check=True) -> int:
    st = lib().pz_kv_amax_update(_ptr(k), _ptr(v), int(n_elems), _ptr(amax), _stream(stream))
    if check and st != 0:
        raise PzError(st, "pz_kv_amax_update")
    return st


def pz_kv_scales_from_amax(amax, round_up_pow2, scales, stream=None, check=True) -> int:
    st = lib().pz_kv_scales_from_amax(_ptr(amax), int(bool(round_up_pow2)), _ptr(scales), _stream(stream))
    if check and st != 0:
        raise PzError(st, "pz_kv_scales_from_amax")
    return st


def pz_window_pages(window, page_size) -> int:
    return int(lib().pz_window_pages(int(window), int(page_size)))


class PagePool:
    """Thin handle on a pz_page_pool (host-side page allocator with window recycling)."""

    def __init__(self, num_pages, page_size, max_seqs, max_pages_per_seq, window=0):
        self._h = lib().pz_page_pool_create(int(num_pages), int(page_size), int(max_seqs), int(max_pages_per_seq),
                                            int(window))
        if not self._h:
            raise PzError(-2, "pz_page_pool_create")
        self.shape = (int(max_seqs), int(max_pages_per_seq))

    def close(self):
        if self._h:
            lib().pz_page_pool_destroy(self._h)
            self._h = None

    __del__ = close

    def append(self, seq, check=True) -> int:
        slot = int(lib().pz_page_pool_append(self._h, int(seq)))
        if check and slot < 0:
            raise PzError(slot, "pz_page_pool_append")
        return slot

    def release(self, seq):
        st = lib().pz_page_pool_release(self._h, int(seq))
        if st != 0:
            raise PzError(st, "pz_page_pool_release")

    def seq_len(self, seq) -> int:
        return int(lib().pz_page_pool_seq_len(self._h, int(seq)))

    def free_pages(self) -> int:
        return int(lib().pz_page_pool_free_pages(self._h))

    def block_table(self):
        """numpy view [max_seqs][max_pages_per_seq] of the pool's host table (valid until close)."""
        import numpy as np
        ptr = lib().pz_page_pool_block_table(self._h)
        return np.ctypeslib.as_array(ptr, shape=self.shape)

    def drain_updates(self):
        """(flat indices, values) of the block-table entries that changed since the last drain."""
        import numpy as np
        n = int(lib().pz_page_pool_pending_updates(self._h))
        idx = np.empty(n, dtype=np.int32)
        val = np.empty(n, dtype=np.int32)
        got = lib().pz_page_pool_drain_updates(self._h, idx.ctypes.data, val.ctypes.data, n) if n else 0
        assert got == n
        return idx, val


def pz_rope_yarn_table(params, head_dim, n_pos, check=True):
    """Host tables (cos, sin) as numpy fp32 [n_pos][head_dim/2]."""
    import numpy as np
    cos = np.zeros((n_pos, head_dim // 2), dtype=np.float32)
    sin = np.zeros((n_pos, head_dim // 2), dtype=np.float32)
    st = lib().pz_rope_yarn_table(C.byref(params), int(head_dim), int(n_pos), cos.ctypes.data, sin.ctypes.data)
    if check and st != 0:
        raise PzError(st, "pz_rope_yarn_table")
    return cos, sin


def pz_rope_kv_append_fp8(cache, q_in, q_out, k_new, v_new, positions, cos_tab, sin_tab, slot_mapping, n_tokens,
                          n_q_heads, k_scale, v_scale, stream=None, check=True) -> int:
    st = lib().pz_rope_kv_append_fp8(_cache_ref(cache), _ptr(q_in), _ptr(q_out), _ptr(k_new), _ptr(v_new),
                                     _ptr(positions), _ptr(cos_tab), _ptr(sin_tab), _ptr(slot_mapping), int(n_tokens),
                                     int(n_q_heads), float(k_scale), float(v_scale), _stream(stream))
    if check and st != 0:
        raise PzError(st, "pz_rope_kv_append_fp8")
    return st


def pz_prefill_attn(cache, q, q_start, block_table, max_pages_per_seq, seq_lens, batch, n_q_heads, max_new_tokens,
                    sinks, sm_scale, k_scale, v_scale, window, out, out_dtype=OUT_F32, stream=None, check=True) -> int:
    st = lib().pz_prefill_attn(_cache_ref(cache), _ptr(q), _ptr(q_start), _ptr(block_table), int(max_pages_per_seq),
                               _ptr(seq_lens), int(batch), int(n_q_heads), int(max_new_tokens), _ptr(sinks),
                               float(sm_scale), float(k_scale), float(v_scale), int(window), _ptr(out), int(out_dtype),
                               _stream(stream))
    if check and st != 0:
        raise PzError(st, "pz_prefill_attn")
    return st
