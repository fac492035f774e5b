"""Seeded synthetic inputs for the decode-attention path (shared by tests, bench and smoke).

This module only *generates inputs*: random tensors, ragged lengths, block tables, slot
mappings, the layer pattern.  It holds none of the method's arithmetic (no FP8 codec, no
attention) and imports neither the oracle nor the HIP binding.  bf16 tensors are carried as
uint16 bit patterns so that the oracle and the GPU path receive the same bytes.

Shapes follow the gpt-oss attention geometry the paper's serving scenarios run on (64 query
heads, 8 KV heads, head_dim 64; alternating window-128 / full layers, 8 of the 18 full layers
turned into window-8192 -- paper Section 2, "Window attention for long-context inference").
The paper's activations come from a real model on its own dataset; N(0,1) data stands in.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

E4M3_MAX = 448.0


# ------------------------------------------------------------------ bf16 plumbing

def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u >> 16                                        # one temporary, updated in place
    r &= np.uint32(1)
    r += np.uint32(0x7FFF)
    r += u
    r >>= 16
    return r.astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def amax_scale(bits: np.ndarray) -> float:
    """Max-calibrated per-tensor scale of the configs: amax / 448, one fp32 divide."""
    amax = np.float32(np.max(np.abs(bf16_to_f32(bits)))) if bits.size else np.float32(0.0)
    s = np.float32(amax) / np.float32(E4M3_MAX)
    return float(s) if s > 0 else 1.0


# ------------------------------------------------------------------ a decode-attention case

@dataclass
class Case:
    name: str
    B: int
    Hq: int
    Hkv: int
    d: int
    P: int
    window: int
    sm_scale: float
    seq_lens: np.ndarray                 # int32 [B], includes the token appended this step
    q: np.ndarray                        # uint16 [B][Hq][d]
    k: np.ndarray                        # uint16 [sum L][Hkv][d], sequences concatenated
    v: np.ndarray                        # uint16 [sum L][Hkv][d]
    sinks: Optional[np.ndarray]          # fp32 [Hq] or None
    k_scale: float
    v_scale: float
    num_pages: int
    block_table: np.ndarray              # int32 [B][max_pages]
    slot_mapping: np.ndarray             # int64 [sum L]: slot of every context token
    split_tokens: int = 0
    extra: dict = field(default_factory=dict)

    @property
    def max_pages(self) -> int:
        return int(self.block_table.shape[1])

    @property
    def offsets(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.seq_lens.astype(np.int64))])


def paged_tables(rng: np.random.Generator, seq_lens: np.ndarray, P: int, spare_pages: int = 2,
                 min_max_pages: int = 1, first_pos=None):
    """Random page assignment: a permutation of the physical pages, dealt to the sequences.

    Returns (num_pages, block_table int32 [B][max_pages], slot_mapping int64 [sum (L - first_pos)]).
    Only the pages that hold positions [first_pos_b, L_b) exist (first_pos_b a multiple of P,
    default 0: the whole context); every other block-table entry holds -1; `spare_pages` pages
    belong to no sequence.  The slot mapping lists the resident positions, sequence by sequence."""
    seq_lens = np.asarray(seq_lens, dtype=np.int64)
    first_pos = np.zeros_like(seq_lens) if first_pos is None else np.asarray(first_pos, dtype=np.int64)
    assert np.all(first_pos % P == 0) and np.all(first_pos <= seq_lens)
    end_page = (seq_lens + P - 1) // P
    n_pages = end_page - first_pos // P
    total = int(n_pages.sum())
    num_pages = total + spare_pages
    perm = rng.permutation(num_pages).astype(np.int32)
    max_pages = max(int(end_page.max(initial=0)), min_max_pages)
    bt = np.full((len(seq_lens), max_pages), -1, dtype=np.int32)
    slots = np.empty(int((seq_lens - first_pos).sum()), dtype=np.int64)
    at, tok = 0, 0
    for b, L in enumerate(seq_lens):
        n, p0 = int(n_pages[b]), int(first_pos[b]) // P
        bt[b, p0:p0 + n] = perm[at:at + n]
        at += n
        j = np.arange(int(first_pos[b]), int(L), dtype=np.int64)
        slots[tok:tok + len(j)] = bt[b, j // P].astype(np.int64) * P + j % P
        tok += len(j)
    return num_pages, bt, slots


def make_case(name: str, *, B: int, Hq: int, Hkv: int, d: int, P: int, seq_lens, window: int = 0,
              seed: int = 0, sinks: bool = True, sm_scale: Optional[float] = None,
              split_tokens: int = 0, outlier_frac: float = 0.0, outlier_gain: float = 20.0,
              pow2_scales: bool = False, unit_scales: bool = False, k_gain: float = 1.0,
              v_gain: float = 1.0) -> Case:
    """q, k, v ~ N(0,1) rounded to bf16; sinks ~ N(0,1) fp32; scales = amax/448 per tensor.

    k_gain / v_gain multiply K / V before the rounding to bf16 (layers of a model differ in the magnitude
    of their activations, hence in their calibrated scales).

    outlier_frac > 0 multiplies round(outlier_frac * Hkv * d) seeded (kv-head, channel) pairs of
    K by `outlier_gain` for every token before calibration (outlier channels)."""
    rng = np.random.default_rng(seed)
    seq_lens = np.asarray(seq_lens, dtype=np.int32)
    assert seq_lens.shape == (B,)
    T = int(seq_lens.astype(np.int64).sum())
    q = rng.standard_normal((B, Hq, d), dtype=np.float32)
    k = rng.standard_normal((T, Hkv, d), dtype=np.float32)
    v = rng.standard_normal((T, Hkv, d), dtype=np.float32)
    if k_gain != 1.0:
        k *= np.float32(k_gain)
    if v_gain != 1.0:
        v *= np.float32(v_gain)
    extra = {}
    if outlier_frac > 0:
        n_out = int(round(outlier_frac * Hkv * d))
        pairs = rng.choice(Hkv * d, size=n_out, replace=False)
        k.reshape(T, Hkv * d)[:, pairs] *= np.float32(outlier_gain)
        extra["outlier_pairs"] = pairs
    sk = rng.standard_normal(Hq).astype(np.float32) if sinks else None
    qb, kb, vb = bf16_bits(q), bf16_bits(k), bf16_bits(v)
    k_scale, v_scale = amax_scale(kb), amax_scale(vb)
    if pow2_scales:                       # exact: frexp/ldexp only
        def up(s):
            m, e = np.frexp(np.float32(s))
            return float(s) if m == 0.5 else float(np.ldexp(np.float32(1.0), e))
        k_scale, v_scale = up(k_scale), up(v_scale)
    if unit_scales:
        k_scale = v_scale = 1.0
    num_pages, bt, slots = paged_tables(rng, seq_lens, P)
    return Case(name=name, B=B, Hq=Hq, Hkv=Hkv, d=d, P=P, window=window,
                sm_scale=float(sm_scale if sm_scale is not None else 1.0 / np.sqrt(d)),
                seq_lens=seq_lens, q=qb, k=kb, v=vb, sinks=sk, k_scale=k_scale, v_scale=v_scale,
                num_pages=num_pages, block_table=bt, slot_mapping=slots, split_tokens=split_tokens,
                extra=extra)


# ------------------------------------------------------------------ the benchmark configurations

def config1_tiny(seed: int = 0) -> Case:
    """Tiny oracle case: batch 2, 8 q / 2 KV heads, d 64, contexts 100 and 37, page size 16."""
    return make_case("cfg1_tiny", B=2, Hq=8, Hkv=2, d=64, P=16, seq_lens=[100, 37], seed=seed,
                     sm_scale=1.0 / 8.0)


def config2_full(seed: int = 2, B: int = 64, L: int = 8192) -> Case:
    """gpt-oss-shaped full-attention layer, every sequence at context L, page size 64."""
    return make_case("cfg2_full", B=B, Hq=64, Hkv=8, d=64, P=64, seq_lens=[L] * B, seed=seed)


def config3_long(seed: int = 3, B: int = 16, L: int = 65536, split_tokens: int = 1024) -> Case:
    """Long-context split-K layer with 1 % outlier K channels (x20) before calibration."""
    return make_case("cfg3_long", B=B, Hq=64, Hkv=8, d=64, P=64, seq_lens=[L] * B, seed=seed,
                     split_tokens=split_tokens, outlier_frac=0.01)


def ragged_lengths(seed: int, B: int, lo: int, hi: int) -> np.ndarray:
    return np.random.default_rng(seed).integers(lo, hi + 1, size=B).astype(np.int32)


def config4_window(seed: int = 4, B: int = 256, window: int = 128, lo: int = 1024,
                   hi: int = 65536) -> Case:
    """Sliding-window layer over ragged contexts uniform in [lo, hi]."""
    return make_case("cfg4_window%d" % window, B=B, Hq=64, Hkv=8, d=64, P=64,
                     seq_lens=ragged_lengths(seed, B, lo, hi), window=window, seed=seed)


def layer_pattern(seed: int = 5, n_layers: int = 36, n_converted: int = 8) -> list:
    """Per-layer window of the heterogeneous model: even layers window 128, odd layers full,
    and `n_converted` seeded odd layers turned into window 8192 (0 = full attention)."""
    full_layers = [i for i in range(n_layers) if i % 2 == 1]
    conv = set(np.random.default_rng(seed).choice(full_layers, size=n_converted, replace=False).tolist())
    return [128 if i % 2 == 0 else (8192 if i in conv else 0) for i in range(n_layers)]


def kv_tokens_read(seq_lens, window: int) -> int:
    """Number of cached tokens one layer's attention reads: sum_b min(L_b, W or inf)."""
    L = np.asarray(seq_lens, dtype=np.int64)
    return int((np.minimum(L, window) if window > 0 else L).sum())


def kv_bytes_per_token(Hkv: int = 8, d: int = 64, elem_bytes: int = 1) -> int:
    """K and V bytes of one cached token of one layer."""
    return 2 * Hkv * d * elem_bytes


# ------------------------------------------------------------------ full-size inputs, generated on the device

@dataclass
class DeviceLayer:
    """One layer's decode inputs resident on the GPU (torch tensors), plus host-side metadata.

    k_ctx / v_ctx (bf16 [sum L][Hkv][d]) are kept only when `keep_context` was asked for; the
    benchmark drops them after the cache has been built."""
    B: int
    Hq: int
    Hkv: int
    d: int
    P: int
    window: int
    sm_scale: float
    seq_lens: np.ndarray
    k_scale: float
    v_scale: float
    num_pages: int
    block_table_host: np.ndarray
    slot_mapping_host: np.ndarray
    q: object
    sinks: object
    block_table: object
    seq_lens_dev: object
    new_slots: object                     # int64 [B]: slot of each sequence's last (new) token
    k_new: object                         # bf16 [B][Hkv][d]: the new token's K rows
    v_new: object
    first_pos: np.ndarray = None          # int64 [B]: first resident position of each sequence
    ctx_offsets: np.ndarray = None        # int64 [B+1]: row offsets of the sequences in k_ctx / v_ctx
    k_ctx: object = None                  # bf16 [sum (L - first_pos)][Hkv][d]: the resident positions
    v_ctx: object = None


def device_layer(*, B, Hq=64, Hkv=8, d=64, P=64, seq_lens, window=0, seed=0, outlier_frac=0.0,
                 outlier_gain=20.0, device="cuda", resident=None):
    """Device-side twin of make_case for sizes that do not fit a host round trip comfortably.

    Same recipe (N(0,1) -> bf16, sinks ~ N(0,1), outlier channels, amax/448 scales, random page
    permutation), drawn from torch's seeded device generator instead of numpy's, so the values
    differ from make_case's but the distribution and structure are the same.  The caller appends
    k_ctx / v_ctx through the library and hands sampled sequences to the oracle.

    resident: keep only the pages that hold the last `resident` positions of every sequence (a
    window layer's cache is bounded by its window); None keeps the whole context."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    rng = np.random.default_rng(seed)
    seq_lens = np.asarray(seq_lens, dtype=np.int32)
    L64 = seq_lens.astype(np.int64)
    first_pos = np.zeros(B, dtype=np.int64) if resident is None else (np.maximum(L64 - resident, 0) // P) * P
    T = int((L64 - first_pos).sum())
    q = torch.randn((B, Hq, d), generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    sinks = torch.randn((Hq,), generator=g, device=device, dtype=torch.float32)
    k = torch.empty((T, Hkv, d), dtype=torch.bfloat16, device=device)
    v = torch.empty((T, Hkv, d), dtype=torch.bfloat16, device=device)
    gain = torch.ones((Hkv * d,), dtype=torch.float32, device=device)
    if outlier_frac > 0:
        pairs = rng.choice(Hkv * d, size=int(round(outlier_frac * Hkv * d)), replace=False)
        gain[torch.from_numpy(pairs).to(device)] = outlier_gain
    gain = gain.view(1, Hkv, d)
    step = 1 << 18
    for t0 in range(0, T, step):
        n = min(step, T - t0)
        k[t0:t0 + n] = (torch.randn((n, Hkv, d), generator=g, device=device) * gain).to(torch.bfloat16)
        v[t0:t0 + n] = torch.randn((n, Hkv, d), generator=g, device=device).to(torch.bfloat16)
    k_amax = float(k.abs().max().float().item()) if T else 0.0
    v_amax = float(v.abs().max().float().item()) if T else 0.0
    k_scale = float(np.float32(k_amax) / np.float32(E4M3_MAX)) or 1.0
    v_scale = float(np.float32(v_amax) / np.float32(E4M3_MAX)) or 1.0
    num_pages, bt, slots = paged_tables(rng, seq_lens, P, first_pos=first_pos)
    ctx_offsets = np.concatenate([[0], np.cumsum(L64 - first_pos)])
    last = ctx_offsets[1:] - 1
    last_dev = torch.from_numpy(last).to(device)
    return DeviceLayer(first_pos=first_pos, ctx_offsets=ctx_offsets, B=B, Hq=Hq, Hkv=Hkv, d=d, P=P, window=window, sm_scale=float(1.0 / np.sqrt(d)),
                       seq_lens=seq_lens, k_scale=k_scale, v_scale=v_scale, num_pages=num_pages,
                       block_table_host=bt, slot_mapping_host=slots, q=q, sinks=sinks,
                       block_table=torch.from_numpy(bt).to(device),
                       seq_lens_dev=torch.from_numpy(seq_lens).to(device),
                       new_slots=torch.from_numpy(slots[last]).to(device),
                       k_new=k[last_dev].contiguous(), v_new=v[last_dev].contiguous(), k_ctx=k, v_ctx=v)
