"""GPU-side test helpers: build caches and run attention through the C ABI binding."""
import numpy as np
import torch

import paper_2602_11937_amd as pz
from workloads import Case

DEV = "cuda"


def dev_bits(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> device int16 tensor with the same bytes."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(DEV)


def gpu_cache(case: Case, dtype=pz.KV_FP8, fill=0xAA, slots=None, k_scale=None, v_scale=None):
    """Canary-filled device cache with every context token appended by pz_kv_append_fp8."""
    cache = pz.PagedCache.allocate(case.num_pages, case.P, case.Hkv, case.d, dtype, DEV,
                                   fill=fill if dtype == pz.KV_FP8 else (fill | (fill << 8)) - 65536)
    slots = case.slot_mapping if slots is None else slots
    k, v = dev_bits(case.k), dev_bits(case.v)
    sm = torch.from_numpy(np.ascontiguousarray(slots, dtype=np.int64)).to(DEV)
    pz.pz_kv_append_fp8(cache, k, v, sm, len(slots), case.k_scale if k_scale is None else k_scale,
                        case.v_scale if v_scale is None else v_scale)
    torch.cuda.synchronize()
    return cache


def to_oracle_layout(cache):
    """Device cache -> host arrays in the oracle's [slot][Hkv][d] layout."""
    k = cache.k.permute(0, 2, 1, 3).contiguous().cpu().numpy()       # [page][P][g][d]
    v = cache.v.permute(0, 3, 1, 2).contiguous().cpu().numpy()       # [page][P][g][d]
    dt = np.uint8 if cache.dtype == pz.KV_FP8 else np.uint16
    shape = (cache.num_pages * cache.page_size, cache.n_kv_heads, cache.head_dim)
    return k.view(dt).reshape(shape), v.view(dt).reshape(shape)


def gpu_attn(case: Case, cache, window=None, split_tokens=0, sinks="case", out_dtype=pz.OUT_F32,
             seq_lens=None, k_scale=None, v_scale=None, sm_scale=None, n_splits=None, return_ws=False,
             q=None):
    window = case.window if window is None else window
    sinks = case.sinks if isinstance(sinks, str) else sinks
    seq_lens = case.seq_lens if seq_lens is None else np.asarray(seq_lens, dtype=np.int32)
    k_scale = case.k_scale if k_scale is None else k_scale
    v_scale = case.v_scale if v_scale is None else v_scale
    sm_scale = case.sm_scale if sm_scale is None else sm_scale
    qd = dev_bits(case.q if q is None else q)
    bt = torch.from_numpy(case.block_table).to(DEV)
    sl = torch.from_numpy(seq_lens).to(DEV)
    sk = None if sinks is None else torch.from_numpy(np.asarray(sinks, dtype=np.float32)).to(DEV)
    tdt = torch.float32 if out_dtype == pz.OUT_F32 else torch.bfloat16
    out = torch.full((case.B, case.Hq, case.d), float("nan"), dtype=tdt, device=DEV)
    ws, wsb, S = None, 0, 0
    if split_tokens > 0:
        S = n_splits or pz.pz_decode_attn_n_splits(int(seq_lens.max(initial=0)), window, split_tokens)
        wsb = pz.pz_decode_attn_workspace_bytes(case.B, case.Hq, case.d, S)
        ws = torch.full((wsb // 4,), float("nan"), dtype=torch.float32, device=DEV)
    pz.pz_decode_attn(cache, qd, bt, case.max_pages, sl, case.B, case.Hq, sk, sm_scale, k_scale, v_scale,
                      window, split_tokens, S, ws, wsb, out, out_dtype)
    if split_tokens > 0:
        pz.pz_decode_attn_splitk_reduce(ws, wsb, case.B, case.Hq, case.d, S, sl, window, split_tokens, sk,
                                        v_scale, out, out_dtype)
    torch.cuda.synchronize()
    res = out.float().cpu().numpy()
    if return_ws:
        w = ws.cpu().numpy()
        n_acc = case.B * case.Hq * S * case.d
        return res, w[:n_acc].reshape(case.B, case.Hq, S, case.d), w[n_acc:].reshape(case.B, case.Hq, S, 2)
    return res
