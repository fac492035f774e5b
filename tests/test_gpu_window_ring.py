"""A decode loop on a sliding-window layer whose cache is bounded by the page pool: every step
appends one token per sequence through recycled pages and attends; the oracle keeps the whole
history in an unbounded cache.  Outputs must agree because positions before the window are never
attended (paper Section 2, "Window attention for long-context inference")."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_11937_amd as pz
from gpu_helpers import DEV, dev_bits
from helpers import rel_err
from workloads import bf16_bits

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("W,P,split", [(20, 16, 0), (128, 64, 0), (300, 64, 128)])
def test_bounded_window_cache_decode_loop(W, P, split):
    B, Hq, Hkv, d, steps = 3, 16, 2, 64, 3 * W + 70
    rng = np.random.default_rng(W)
    k_all = bf16_bits(rng.standard_normal((steps, B, Hkv, d)).astype(np.float32))
    v_all = bf16_bits(rng.standard_normal((steps, B, Hkv, d)).astype(np.float32))
    sinks = rng.standard_normal(Hq).astype(np.float32)
    k_scale = v_scale = 5.0 / 448
    per_seq = pz.pz_window_pages(W, P)
    max_pages = steps // P + 1
    pool = pz.PagePool(B * per_seq, P, B, max_pages, window=W)       # far fewer pages than the history needs
    assert B * per_seq < B * max_pages
    cache = pz.PagedCache.allocate(B * per_seq, P, Hkv, d, pz.KV_FP8, DEV, fill=0x7F)   # NaN codes everywhere
    bt_dev = torch.full((B, max_pages), -1, dtype=torch.int32, device=DEV)
    # the oracle: unbounded cache, sequence b owns pages b*max_pages ...
    okc, ovc = oracle.new_cache(B * max_pages * P, Hkv, d)
    obt = (np.arange(B)[:, None] * max_pages + np.arange(max_pages)[None, :]).astype(np.int32)
    sd = torch.from_numpy(sinks).to(DEV)
    checked = 0
    for t in range(steps):
        slots = np.array([pool.append(b) for b in range(B)], dtype=np.int64)
        idx, val = pool.drain_updates()
        if len(idx):
            bt_dev.view(-1)[torch.from_numpy(idx.astype(np.int64)).to(DEV)] = torch.from_numpy(val).to(DEV)
        pz.pz_kv_append_fp8(cache, dev_bits(k_all[t]), dev_bits(v_all[t]), torch.from_numpy(slots).to(DEV), B,
                            k_scale, v_scale)
        oslots = obt[np.arange(B), t // P].astype(np.int64) * P + t % P
        oracle.kv_append(okc, ovc, k_all[t], v_all[t], oslots, k_scale, v_scale)
        if t % 37 and t != steps - 1 and t not in (W - 1, W, W + 1, 2 * W):
            continue
        q = bf16_bits(rng.standard_normal((B, Hq, d)).astype(np.float32))
        lens = np.full(B, t + 1, dtype=np.int32)
        out = torch.full((B, Hq, d), float("nan"), device=DEV)
        ws, wsb, S = None, 0, 0
        if split:
            S = pz.pz_decode_attn_n_splits(t + 1, W, split)
            wsb = pz.pz_decode_attn_workspace_bytes(B, Hq, d, S)
            ws = torch.full((wsb // 4,), float("nan"), device=DEV)
        sl = torch.from_numpy(lens).to(DEV)
        pz.pz_decode_attn(cache, dev_bits(q), bt_dev, max_pages, sl, B, Hq, sd, 0.125, k_scale, v_scale, W, split, S,
                          ws, wsb, out)
        if split:
            pz.pz_decode_attn_splitk_reduce(ws, wsb, B, Hq, d, S, sl, W, split, sd, v_scale, out)
        torch.cuda.synchronize()
        want = oracle.decode_attn(okc, ovc, P, q, obt, lens, sinks, 0.125, k_scale, v_scale, W, accum="f64")
        got = out.cpu().numpy()
        assert not np.any(np.isnan(got)) and rel_err(got, want) <= 2e-3, t
        checked += 1
    assert checked >= 8 and pool.free_pages() >= 0
    held = (pool.block_table() >= 0).sum(axis=1)
    assert np.all(held <= per_seq)
    pool.close()
