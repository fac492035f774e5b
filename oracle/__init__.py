"""ctypes front end of the CPU oracle (oracle/pz_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package.
It shares nothing with the HIP path and never imports it.  All arrays are numpy arrays on the
host; bf16 tensors travel as uint16 bit patterns.

Oracle cache layout: [num_slots][Hkv][d], slot = physical_page * P + offset (see pz_oracle.c).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pz_oracle.c")
_LIB = os.path.join(_HERE, "libpz_oracle.so")
CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra", "-shared", "-fPIC"]

KV_FP8, KV_BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (rebuilds when the source is newer than the library)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm", "-lpthread"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        # PZ_ORACLE_LIB: load this prebuilt oracle library instead (the test that plants mistakes into
        # copies of pz_oracle.c runs the pins against those copies this way)
        L = C.CDLL(os.environ.get("PZ_ORACLE_LIB") or build())
        L.pzo_bf16_to_f32.restype = C.c_float
        L.pzo_bf16_to_f32.argtypes = [C.c_uint16]
        L.pzo_f32_to_bf16.restype = C.c_uint16
        L.pzo_f32_to_bf16.argtypes = [C.c_float]
        L.pzo_e4m3_decode.restype = C.c_float
        L.pzo_e4m3_decode.argtypes = [C.c_uint8]
        L.pzo_e4m3_encode.restype = C.c_uint8
        L.pzo_e4m3_encode.argtypes = [C.c_float]
        L.pzo_quantize.restype = C.c_uint8
        L.pzo_quantize.argtypes = [C.c_uint16, C.c_float]
        L.pzo_round_scale_up_pow2.restype = C.c_float
        L.pzo_round_scale_up_pow2.argtypes = [C.c_float]
        L.pzo_yarn_table.restype = None
        L.pzo_yarn_table.argtypes = [C.c_double, C.c_double, C.c_int, C.c_double, C.c_double, C.c_int, C.c_int,
                                     C.c_void_p, C.c_void_p]
        L.pzo_rope_kv_append.restype = None
        L.pzo_rope_kv_append.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                         C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_int64, C.c_float, C.c_float]
        L.pzo_amax_bf16.restype = C.c_float
        L.pzo_amax_bf16.argtypes = [C.c_void_p, C.c_int64]
        L.pzo_scale_from_amax.restype = C.c_float
        L.pzo_scale_from_amax.argtypes = [C.c_float, C.c_int]
        L.pzo_kv_append.restype = None
        L.pzo_kv_append.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.c_int64, C.c_float, C.c_float]
        L.pzo_decode_attn.restype = None
        L.pzo_decode_attn.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int,
                                      C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                      C.c_void_p, C.c_float, C.c_float, C.c_float, C.c_int, C.c_int,
                                      C.c_void_p, C.c_int64, C.c_void_p, C.c_int]
        L.pzo_decode_attn_partials.restype = None
        L.pzo_decode_attn_partials.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int,
                                               C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p,
                                               C.c_int, C.c_int, C.c_float, C.c_float, C.c_int,
                                               C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                               C.c_int]
        L.pzo_splitk_reduce.restype = None
        L.pzo_splitk_reduce.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int,
                                        C.c_void_p, C.c_float, C.c_void_p]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _req(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


# ---------------------------------------------------------------- scalar codec helpers

def e4m3_decode(codes) -> np.ndarray:
    codes = np.asarray(codes, dtype=np.uint8)
    f = lib().pzo_e4m3_decode
    return np.array([f(int(c)) for c in codes.ravel()], dtype=np.float32).reshape(codes.shape)


def e4m3_encode(x) -> np.ndarray:
    x = np.asarray(x, dtype=np.float32)
    f = lib().pzo_e4m3_encode
    return np.array([f(float(v)) for v in x.ravel()], dtype=np.uint8).reshape(x.shape)


def quantize(x_bf16_bits, scale: float) -> np.ndarray:
    x = np.asarray(x_bf16_bits, dtype=np.uint16)
    f = lib().pzo_quantize
    return np.array([f(int(v), float(scale)) for v in x.ravel()], dtype=np.uint8).reshape(x.shape)


def bf16_to_f32(bits) -> np.ndarray:
    bits = np.asarray(bits, dtype=np.uint16)
    f = lib().pzo_bf16_to_f32
    return np.array([f(int(v)) for v in bits.ravel()], dtype=np.float32).reshape(bits.shape)


def f32_to_bf16(x) -> np.ndarray:
    x = np.asarray(x, dtype=np.float32)
    f = lib().pzo_f32_to_bf16
    return np.array([f(float(v)) for v in x.ravel()], dtype=np.uint16).reshape(x.shape)


def round_scale_up_pow2(s: float) -> float:
    return float(lib().pzo_round_scale_up_pow2(float(s)))


def yarn_table(d, n_pos, theta=150000.0, factor=56.0, original_context=4096, beta_fast=32.0, beta_slow=1.0):
    """(cos, sin) fp32 [n_pos][d/2] of YaRN-scaled rotary embedding, temperature folded in."""
    cos = np.zeros((n_pos, d // 2), dtype=np.float32)
    sin = np.zeros((n_pos, d // 2), dtype=np.float32)
    lib().pzo_yarn_table(float(theta), float(factor), int(original_context), float(beta_fast), float(beta_slow),
                         int(d), int(n_pos), _p(cos), _p(sin))
    return cos, sin


def rope_kv_append(k_cache, v_cache, q_bits, k_new_bits, v_new_bits, positions, cos_tab, sin_tab, slot_mapping,
                   k_scale, v_scale) -> np.ndarray:
    """Fused rotary + append by the definition; returns the rotated q (bf16 bits [T][Hq][d])."""
    kv_dtype = KV_FP8 if k_cache.dtype == np.uint8 else KV_BF16
    _, Hkv, d = k_cache.shape
    q = _req(q_bits, np.uint16)
    T, Hq, _ = q.shape
    k_new, v_new = _req(k_new_bits, np.uint16), _req(v_new_bits, np.uint16)
    pos, slots = _req(positions, np.int32), _req(slot_mapping, np.int64)
    ct, st = _req(cos_tab, np.float32), _req(sin_tab, np.float32)
    assert k_new.shape == (T, Hkv, d) and pos.shape == (T,) and slots.shape == (T,)
    assert ct.shape == st.shape and ct.shape[1] == d // 2 and pos.max(initial=0) < ct.shape[0]
    q_out = np.zeros_like(q)
    lib().pzo_rope_kv_append(_p(k_cache), _p(v_cache), kv_dtype, Hkv, Hq, d, _p(q), _p(q_out), _p(k_new), _p(v_new),
                             _p(pos), _p(ct), _p(st), _p(slots), T, float(k_scale), float(v_scale))
    return q_out


def amax_bf16(bits) -> float:
    """Largest magnitude of a bf16 tensor (NaN ignored, empty -> 0)."""
    x = _req(bits, np.uint16)
    return float(lib().pzo_amax_bf16(_p(x), x.size))


def scale_from_amax(amax: float, round_up_pow2: bool = False) -> float:
    return float(lib().pzo_scale_from_amax(float(amax), int(bool(round_up_pow2))))


# ---------------------------------------------------------------- cache + attention

def new_cache(num_slots: int, Hkv: int, d: int, kv_dtype: int = KV_FP8, fill: int = 0xAA):
    """K and V caches in the oracle layout, pre-filled with a canary byte."""
    dt = np.uint8 if kv_dtype == KV_FP8 else np.uint16
    fillv = fill if kv_dtype == KV_FP8 else (fill | (fill << 8))
    k = np.full((num_slots, Hkv, d), fillv, dtype=dt)
    v = np.full((num_slots, Hkv, d), fillv, dtype=dt)
    return k, v


def kv_append(k_cache, v_cache, k_new_bits, v_new_bits, slot_mapping, k_scale, v_scale):
    """Quantise (or copy, for a bf16 cache) new K/V rows into the cache, in place."""
    kv_dtype = KV_FP8 if k_cache.dtype == np.uint8 else KV_BF16
    assert k_cache.flags.c_contiguous and v_cache.flags.c_contiguous
    _, Hkv, d = k_cache.shape
    k_new = _req(k_new_bits, np.uint16)
    v_new = _req(v_new_bits, np.uint16)
    slots = _req(slot_mapping, np.int64)
    T = slots.shape[0]
    assert k_new.shape == (T, Hkv, d) and v_new.shape == (T, Hkv, d)
    assert slots.max(initial=-1) < k_cache.shape[0]
    lib().pzo_kv_append(_p(k_cache), _p(v_cache), kv_dtype, Hkv, d, _p(k_new), _p(v_new), _p(slots),
                        T, float(k_scale), float(v_scale))


def _check_tables(k_cache, P, block_table, seq_lens, window=0):
    """Every page that holds an attended position must be a valid physical page."""
    B, max_pages = block_table.shape
    assert seq_lens.shape == (B,)
    num_pages = k_cache.shape[0] // P
    for b in range(B):
        L = int(seq_lens[b])
        n = -(-L // P)
        assert n <= max_pages
        if n:
            lo = L - window if (window > 0 and L > window) else 0
            used = block_table[b, lo // P:n]
            assert 0 <= used.min() and used.max() < num_pages


def decode_attn(k_cache, v_cache, P, q_bits, block_table, seq_lens, sinks, sm_scale, k_scale,
                v_scale, window=0, accum="f32", rows=None, nthreads=1) -> np.ndarray:
    """Unsplit decode attention by the definition; returns fp32 [B][Hq][d].

    rows: optional int array of b*Hq+h; other rows of the result stay zero."""
    kv_dtype = KV_FP8 if k_cache.dtype == np.uint8 else KV_BF16
    _, Hkv, d = k_cache.shape
    q = _req(q_bits, np.uint16)
    B, Hq, dq = q.shape
    assert dq == d and Hq % Hkv == 0
    bt = _req(block_table, np.int32)
    sl = _req(seq_lens, np.int32)
    _check_tables(k_cache, P, bt, sl, window)
    sk = None if sinks is None else _req(sinks, np.float32)
    out = np.zeros((B, Hq, d), dtype=np.float32)
    r = None if rows is None else _req(rows, np.int32)
    lib().pzo_decode_attn(_p(k_cache), _p(v_cache), kv_dtype, P, Hkv, d, _p(q), _p(bt), bt.shape[1],
                          _p(sl), B, Hq, _p(sk), float(sm_scale), float(k_scale), float(v_scale),
                          int(window), 0 if accum == "f32" else 1, _p(r),
                          0 if r is None else r.shape[0], _p(out), int(nthreads))
    return out


def decode_attn_partials(k_cache, v_cache, P, q_bits, block_table, seq_lens, sm_scale, k_scale,
                         window, split_tokens, n_splits, accum="f32", nthreads=1):
    """Sink-free split-K partials by the chunked definition: (acc [B][Hq][S][d], ml [B][Hq][S][2])."""
    kv_dtype = KV_FP8 if k_cache.dtype == np.uint8 else KV_BF16
    _, Hkv, d = k_cache.shape
    q = _req(q_bits, np.uint16)
    B, Hq, _ = q.shape
    bt = _req(block_table, np.int32)
    sl = _req(seq_lens, np.int32)
    _check_tables(k_cache, P, bt, sl, window)
    acc = np.zeros((B, Hq, n_splits, d), dtype=np.float32)
    ml = np.zeros((B, Hq, n_splits, 2), dtype=np.float32)
    lib().pzo_decode_attn_partials(_p(k_cache), _p(v_cache), kv_dtype, P, Hkv, d, _p(q), _p(bt),
                                   bt.shape[1], _p(sl), B, Hq, float(sm_scale), float(k_scale),
                                   int(window), int(split_tokens), int(n_splits),
                                   0 if accum == "f32" else 1, _p(acc), _p(ml), int(nthreads))
    return acc, ml


def splitk_reduce(part_acc, part_ml, sinks, v_scale) -> np.ndarray:
    acc = _req(part_acc, np.float32)
    ml = _req(part_ml, np.float32)
    B, Hq, S, d = acc.shape
    assert ml.shape == (B, Hq, S, 2)
    sk = None if sinks is None else _req(sinks, np.float32)
    out = np.zeros((B, Hq, d), dtype=np.float32)
    lib().pzo_splitk_reduce(_p(acc), _p(ml), B, Hq, d, S, _p(sk), float(v_scale), _p(out))
    return out


def prefill_attn(k_cache, v_cache, P, q_bits, q_start, block_table, seq_lens, sinks, sm_scale, k_scale, v_scale,
                 window=0, accum="f32", nthreads=1) -> np.ndarray:
    """Multi-token attention by the definition: query i of sequence b sits at position
    p = L_b - n_b + i and is, by definition, a decode query against the first p + 1 positions
    (causal), inside the window.  So every query token becomes one row of decode_attn with
    sequence length p + 1 and its sequence's block-table row.  Returns fp32 [T][Hq][d]."""
    q = _req(q_bits, np.uint16)
    qs = np.asarray(q_start, dtype=np.int64)
    bt = _req(block_table, np.int32)
    sl = np.asarray(seq_lens, dtype=np.int64)
    T = q.shape[0]
    assert qs[0] == 0 and qs[-1] == T and len(qs) == len(sl) + 1
    rows_bt = np.empty((T, bt.shape[1]), dtype=np.int32)
    rows_len = np.empty(T, dtype=np.int32)
    for b in range(len(sl)):
        n = int(qs[b + 1] - qs[b])
        assert 0 <= n <= sl[b]
        rows_bt[qs[b]:qs[b + 1]] = bt[b]
        rows_len[qs[b]:qs[b + 1]] = sl[b] - n + np.arange(n) + 1
    return decode_attn(k_cache, v_cache, P, q, rows_bt, rows_len, sinks, sm_scale, k_scale, v_scale, window,
                       accum=accum, nthreads=nthreads)
