"""GPU parity with the pages of a case placed at the top of a cache larger than 4 GiB per tensor:
every byte offset the kernels form from a page id is then above 2^32.  The oracle runs on the
compact case (its result does not depend on which physical pages hold the tokens)."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
import paper_2602_11937_amd as pz
import workloads as wl
from gpu_helpers import DEV, dev_bits, gpu_attn, gpu_cache, to_oracle_layout
from helpers import oracle_cache, rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-3
GIB = 1 << 30


def lifted(case, kv_dtype=pz.KV_FP8):
    """The same case with its pages moved to the end of a cache of more than 4 GiB per tensor."""
    page_bytes = case.Hkv * case.P * case.d * (1 if kv_dtype == pz.KV_FP8 else 2)
    num_big = (4 * GIB + GIB // 4) // page_bytes + case.num_pages
    shift = num_big - case.num_pages
    assert shift * page_bytes > 4 * GIB
    bt = np.where(case.block_table >= 0, case.block_table + shift, -1).astype(np.int32)
    return dataclasses.replace(case, num_pages=num_big, block_table=bt,
                               slot_mapping=case.slot_mapping + np.int64(shift) * case.P), shift


def top_pages(cache, shift):
    return pz.PagedCache(cache.k[shift:], cache.v[shift:], cache.num_pages - shift, cache.page_size,
                         cache.n_kv_heads, cache.head_dim, cache.dtype)


def untouched_below(cache, shift, fill):
    step = 16384
    for a in range(0, shift, step):
        if bool((cache.k[a:min(a + step, shift)] != fill).any()) or bool((cache.v[a:min(a + step, shift)] != fill).any()):
            return False
    return True


@pytest.mark.parametrize("kv_dtype", [pz.KV_FP8, pz.KV_BF16])
def test_append_and_decode_beyond_4_gib(kv_dtype):
    case = wl.make_case("big", B=3, Hq=64, Hkv=8, d=64, P=64, seq_lens=[3000, 700, 65], seed=40)
    big, shift = lifted(case, kv_dtype)
    ks, vs = (case.k_scale, case.v_scale) if kv_dtype == pz.KV_FP8 else (1.0, 1.0)
    cache = gpu_cache(big, dtype=kv_dtype, k_scale=ks, v_scale=vs)
    gk, gv = to_oracle_layout(top_pages(cache, shift))
    okv = oracle.KV_FP8 if kv_dtype == pz.KV_FP8 else oracle.KV_BF16
    ok, ov = oracle_cache(case, okv)
    assert np.array_equal(gk, ok) and np.array_equal(gv, ov)
    assert untouched_below(cache, shift, 0xAA if kv_dtype == pz.KV_FP8 else (0xAAAA - 65536))
    for window, split in ((0, 0), (0, 256), (500, 0), (500, 256)):
        want = oracle.decode_attn(ok, ov, case.P, case.q, case.block_table, case.seq_lens, sinks=case.sinks,
                                  sm_scale=case.sm_scale, k_scale=ks, v_scale=vs, window=window, nthreads=8)
        got = gpu_attn(big, cache, window=window, split_tokens=split, k_scale=ks, v_scale=vs)
        assert not np.any(np.isnan(got)) and rel_err(got, want) <= TOL, (window, split)


def test_128_channel_heads_beyond_4_gib():
    case = wl.make_case("big128", B=3, Hq=16, Hkv=4, d=128, P=64, seq_lens=[3000, 700, 65], seed=42)
    big, shift = lifted(case)
    cache = gpu_cache(big)
    gk, gv = to_oracle_layout(top_pages(cache, shift))
    ok, ov = oracle_cache(case)
    assert np.array_equal(gk, ok) and np.array_equal(gv, ov)
    assert untouched_below(cache, shift, 0xAA)
    for window, split in ((0, 0), (0, 256), (500, 256)):
        want = oracle.decode_attn(ok, ov, case.P, case.q, case.block_table, case.seq_lens, sinks=case.sinks,
                                  sm_scale=case.sm_scale, k_scale=case.k_scale, v_scale=case.v_scale, window=window,
                                  nthreads=8)
        got = gpu_attn(big, cache, window=window, split_tokens=split)
        assert not np.any(np.isnan(got)) and rel_err(got, want) <= TOL, (window, split)


def test_fused_append_rotary_append_and_prefill_beyond_4_gib():
    case = wl.make_case("big2", B=2, Hq=16, Hkv=8, d=64, P=64, seq_lens=[900, 130], seed=41)
    big, shift = lifted(case)
    last = case.offsets[1:] - 1
    prefix = big.slot_mapping.copy()
    prefix[last] = -1
    ok, ov = oracle_cache(case)

    # the newest token of each sequence through the fused call (single pass, then split-K)
    for split in (0, 256):
        cache = gpu_cache(big, slots=prefix)
        S = pz.pz_decode_attn_n_splits(int(case.seq_lens.max()), 0, split) if split else 0
        wsb = pz.pz_decode_attn_workspace_bytes(case.B, case.Hq, case.d, S) if split else 0
        ws = torch.full((max(wsb, 4) // 4,), float("nan"), dtype=torch.float32, device=DEV)
        out = torch.full((case.B, case.Hq, case.d), float("nan"), dtype=torch.float32, device=DEV)
        sl = torch.from_numpy(case.seq_lens).to(DEV)
        sinks = torch.from_numpy(case.sinks).to(DEV)
        pz.pz_decode_attn_append(cache, dev_bits(case.k[last]), dev_bits(case.v[last]), dev_bits(case.q),
                                 torch.from_numpy(big.block_table).to(DEV), big.max_pages, sl, case.B, case.Hq, sinks,
                                 case.sm_scale, case.k_scale, case.v_scale, 0, split, S, ws if split else None, wsb, out)
        if split:
            pz.pz_decode_attn_splitk_reduce(ws, wsb, case.B, case.Hq, case.d, S, sl, 0, split, sinks, case.v_scale, out)
        torch.cuda.synchronize()
        gk, gv = to_oracle_layout(top_pages(cache, shift))
        assert np.array_equal(gk, ok) and np.array_equal(gv, ov)
        want = oracle.decode_attn(ok, ov, case.P, case.q, case.block_table, case.seq_lens, sinks=case.sinks,
                                  sm_scale=case.sm_scale, k_scale=case.k_scale, v_scale=case.v_scale, nthreads=8)
        assert rel_err(out.cpu().numpy(), want) <= TOL, split

    # multi-token attention over the lifted pages
    n_new = [70, 130]
    q_start = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
    rng = np.random.default_rng(41)
    q = wl.bf16_bits(rng.standard_normal((int(q_start[-1]), case.Hq, case.d)).astype(np.float32))
    cache = gpu_cache(big)
    out = torch.full((int(q_start[-1]), case.Hq, case.d), float("nan"), dtype=torch.float32, device=DEV)
    pz.pz_prefill_attn(cache, dev_bits(q), torch.from_numpy(q_start).to(DEV), torch.from_numpy(big.block_table).to(DEV),
                       big.max_pages, torch.from_numpy(case.seq_lens).to(DEV), case.B, case.Hq, max(n_new),
                       torch.from_numpy(case.sinks).to(DEV), case.sm_scale, case.k_scale, case.v_scale, 0, out)
    torch.cuda.synchronize()
    want = oracle.prefill_attn(ok, ov, case.P, q, q_start, case.block_table, case.seq_lens, case.sinks, case.sm_scale,
                               case.k_scale, case.v_scale, 0, accum="f64", nthreads=8)
    assert rel_err(out.cpu().numpy(), want) <= TOL

    # rotary + quantise + append of the whole context into the lifted pages
    T = len(case.slot_mapping)
    positions = np.concatenate([np.arange(L) for L in case.seq_lens]).astype(np.int32)
    cos, sin = pz.pz_rope_yarn_table(pz.YarnParams(), case.d, int(case.seq_lens.max()))
    cache = pz.PagedCache.allocate(big.num_pages, case.P, case.Hkv, case.d, pz.KV_FP8, DEV, fill=0xAA)
    qin = wl.bf16_bits(rng.standard_normal((T, case.Hq, case.d)).astype(np.float32))
    qout = torch.zeros((T, case.Hq, case.d), dtype=torch.int16, device=DEV)
    pz.pz_rope_kv_append_fp8(cache, dev_bits(qin), qout, dev_bits(case.k), dev_bits(case.v),
                             torch.from_numpy(positions).to(DEV), torch.from_numpy(cos).to(DEV),
                             torch.from_numpy(sin).to(DEV), torch.from_numpy(big.slot_mapping).to(DEV), T, case.Hq,
                             case.k_scale, case.v_scale)
    torch.cuda.synchronize()
    rk, rv = oracle.new_cache(case.num_pages * case.P, case.Hkv, case.d)
    want_q = oracle.rope_kv_append(rk, rv, qin, case.k, case.v, positions, cos, sin, case.slot_mapping,
                                   case.k_scale, case.v_scale)
    gk, gv = to_oracle_layout(top_pages(cache, shift))
    assert np.array_equal(gk, rk) and np.array_equal(gv, rv)
    assert np.array_equal(qout.cpu().numpy().view(np.uint16), want_q)
