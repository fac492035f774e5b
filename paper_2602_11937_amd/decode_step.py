"""The per-layer loop of one decode step, on top of the C-ABI binding (marshalling and the loop only).

A model of the paper's kind is a stack of attention layers that differ in two things the library takes
as plain arguments: the attention range -- full context or a sliding window of 128 or 8192 positions,
chosen per layer (paper Section 2, "Window attention for long-context inference") -- and the K and V
scales of the layer's FP8 cache (Section 3, "KV Quantization").  One decode step visits every layer:
quantise-and-append of the one new token per sequence, attention of the new query over the layer's cache
(single pass for short windows, split-K partials + log-sum-exp merge otherwise).  `DecodeLayer` holds what
one layer owns and issues its calls; `DecodeStep` walks the stack with ONE split-K workspace that all
layers share (the calls are enqueued on one stream, so a layer's merge has consumed the workspace before
the next layer's partials are written; rows a layer does not write are never read by its merge).

Everything here enqueues kernels through `binding`; nothing is computed in Python.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Sequence

from . import binding as pz


@dataclass
class DecodeLayer:
    """One attention layer's cache, tables and per-layer constants."""
    cache: pz.PagedCache
    block_table: object                  # device int32 [batch][max_pages]
    max_pages: int
    window: int                          # 0 = full attention
    k_scale: float
    v_scale: float
    sm_scale: float
    sinks: Optional[object]              # device fp32 [n_q_heads] or None
    split_tokens: int = 0                # 0 = single pass, else the split-K chunk length

    def n_splits(self, max_seq_len: int) -> int:
        return pz.pz_decode_attn_n_splits(max_seq_len, self.window, self.split_tokens) if self.split_tokens else 0

    def workspace_bytes(self, batch: int, n_q_heads: int, max_seq_len: int) -> int:
        if not self.split_tokens:
            return 0
        return pz.pz_decode_attn_workspace_bytes(batch, n_q_heads, self.cache.head_dim, self.n_splits(max_seq_len))

    def append(self, k_new, v_new, new_slots, batch, stream=None):
        pz.pz_kv_append_fp8(self.cache, k_new, v_new, new_slots, batch, self.k_scale, self.v_scale, stream)

    def attend(self, q, seq_lens, batch, n_q_heads, n_splits, workspace, workspace_bytes, out, out_dtype=pz.OUT_F32,
               stream=None):
        split = self.split_tokens
        pz.pz_decode_attn(self.cache, q, self.block_table, self.max_pages, seq_lens, batch, n_q_heads, self.sinks,
                          self.sm_scale, self.k_scale, self.v_scale, self.window, split, n_splits,
                          workspace if split else None, workspace_bytes if split else 0, out, out_dtype, stream)

    def attend_append(self, k_new, v_new, q, seq_lens, batch, n_q_heads, n_splits, workspace, workspace_bytes, out,
                      out_dtype=pz.OUT_F32, stream=None):
        split = self.split_tokens
        pz.pz_decode_attn_append(self.cache, k_new, v_new, q, self.block_table, self.max_pages, seq_lens, batch,
                                 n_q_heads, self.sinks, self.sm_scale, self.k_scale, self.v_scale, self.window, split,
                                 n_splits, workspace if split else None, workspace_bytes if split else 0, out,
                                 out_dtype, stream)

    def merge(self, seq_lens, batch, n_q_heads, n_splits, workspace, workspace_bytes, out, out_dtype=pz.OUT_F32,
              stream=None):
        if self.split_tokens:
            pz.pz_decode_attn_splitk_reduce(workspace, workspace_bytes, batch, n_q_heads, self.cache.head_dim, n_splits,
                                            seq_lens, self.window, self.split_tokens, self.sinks, self.v_scale, out,
                                            out_dtype, stream)

    def step(self, q, k_new, v_new, new_slots, seq_lens, batch, n_q_heads, n_splits, workspace, workspace_bytes, out,
             out_dtype=pz.OUT_F32, fused=False, stream=None):
        """Append + attention (+ merge) of this layer: three calls, or two with the append fused."""
        if fused:
            self.attend_append(k_new, v_new, q, seq_lens, batch, n_q_heads, n_splits, workspace, workspace_bytes, out,
                               out_dtype, stream)
        else:
            self.append(k_new, v_new, new_slots, batch, stream)
            self.attend(q, seq_lens, batch, n_q_heads, n_splits, workspace, workspace_bytes, out, out_dtype, stream)
        self.merge(seq_lens, batch, n_q_heads, n_splits, workspace, workspace_bytes, out, out_dtype, stream)


@dataclass
class LayerInputs:
    """What a step hands one layer: the new token's query, K and V rows and the slots they go to."""
    q: object                            # device bf16 [batch][n_q_heads][d]
    k_new: object                        # device bf16 [batch][n_kv_heads][d]
    v_new: object
    new_slots: object                    # device int64 [batch] (not needed by the fused form)
    out: object                          # device [batch][n_q_heads][d]


class DecodeStep:
    """The stack of layers and the workspace they share."""

    def __init__(self, layers: Sequence[DecodeLayer], batch: int, n_q_heads: int, max_seq_len: int, device="cuda"):
        import torch
        self.layers = list(layers)
        self.batch, self.n_q_heads, self.max_seq_len = batch, n_q_heads, max_seq_len
        self.n_splits = [l.n_splits(max_seq_len) for l in self.layers]
        self.ws_bytes = [l.workspace_bytes(batch, n_q_heads, max_seq_len) for l in self.layers]
        self.workspace = torch.empty((max(max(self.ws_bytes, default=0), 4) // 4,), dtype=torch.float32, device=device)

    def run(self, inputs: Sequence[LayerInputs], seq_lens, out_dtype=pz.OUT_F32, fused=False, stream=None):
        """One decode step: every layer in order.  `seq_lens` (device int32 [batch]) counts the new token."""
        for layer, x, S, nbytes in zip(self.layers, inputs, self.n_splits, self.ws_bytes):
            layer.step(x.q, x.k_new, x.v_new, x.new_slots, seq_lens, self.batch, self.n_q_heads, S, self.workspace,
                       nbytes, x.out, out_dtype, fused, stream)
