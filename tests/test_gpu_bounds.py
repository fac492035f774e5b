"""Device-side inputs that the host cannot check (block-table entries, sequence lengths, slots) are
held to the cache and the table by the kernels: page ids are cut to [0, num_pages), lengths to what
a block-table row covers, tokens with a slot outside the cache are skipped.  Such inputs are the
caller's mistake and their rows are meaningless, but every other row must be what the oracle
gives, and no byte of the cache that a valid call would not write may change."""
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
I32_MAX, I32_MIN = 2 ** 31 - 1, -2 ** 31


def hostile(case):
    """Copy of the case in which sequence 1 has page ids outside the cache at attended positions,
    sequence 2 a length far beyond its block-table row and sequence 3 a negative length."""
    bt = case.block_table.copy()
    bad = np.array([-1, case.num_pages, I32_MAX, I32_MIN, case.num_pages + 12345, -77], dtype=np.int32)
    n_attended = (int(case.seq_lens[1]) + case.P - 1) // case.P
    bt[1, :n_attended] = bad[np.arange(n_attended) % len(bad)]
    lens = case.seq_lens.copy()
    lens[2] = 1_000_000_000
    lens[3] = -7
    return dataclasses.replace(case, block_table=bt), lens


ROUTES = {
    "single_pass": dict(split_tokens=0),
    "single_pass_4_waves": dict(split_tokens=0, force={"attn_waves": 4}),
    "split_balanced": dict(split_tokens=64),
    "split_fixed_grid": dict(split_tokens=64, force={"attn_balanced": 0}),
    "split_fixed_grid_chunk_groups": dict(split_tokens=64, force={"attn_balanced": 0, "attn_chunks_per_group": 3}),
    "split_2_waves": dict(split_tokens=128, force={"attn_waves": 2}),
    "window_single_pass": dict(split_tokens=0, window=100),
    "window_split": dict(split_tokens=64, window=200),
}


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("P", [16, 64])
@pytest.mark.parametrize("route", sorted(ROUTES))
def test_attention_with_hostile_tables_and_lengths(route, P, d, launch_override):
    r = ROUTES[route]
    for name, value in r.get("force", {}).items():
        launch_override(name, value)
    window = r.get("window", 0)
    case = wl.make_case("h", B=5, Hq=8, Hkv=2, d=d, P=P, seq_lens=[300, 517, 130, 260, 411], seed=70 + P, window=window)
    cache = gpu_cache(case)
    kc, vc = oracle_cache(case)
    want = oracle.decode_attn(kc, vc, case.P, case.q, case.block_table, case.seq_lens, sinks=case.sinks,
                              sm_scale=case.sm_scale, k_scale=case.k_scale, v_scale=case.v_scale, window=window,
                              nthreads=8)
    bad_case, bad_lens = hostile(case)
    split = r["split_tokens"]
    # the chunk count a caller would derive from the row length, not from the nonsense length
    S = pz.pz_decode_attn_n_splits(case.max_pages * P, window, split) if split else None
    got = gpu_attn(bad_case, cache, window=window, split_tokens=split, seq_lens=bad_lens, n_splits=S)
    for b in (0, 4):                                               # the sequences with valid inputs
        assert rel_err(got[b], want[b]) <= TOL, (route, b)
    assert np.all(got[3] == 0.0)                                   # a negative length is an empty context
    gk, gv = to_oracle_layout(cache)
    assert np.array_equal(gk, kc) and np.array_equal(gv, vc)       # reading never writes


@pytest.mark.parametrize("d", [64, 128])             # 128-channel heads always append by a launch of their own
@pytest.mark.parametrize("way", ["in_kernel", "own_launch"])
@pytest.mark.parametrize("split_tokens", [0, 64])
def test_fused_append_skips_tokens_it_cannot_place(way, split_tokens, d, launch_override):
    launch_override("append_fused", 1 if way == "in_kernel" else 0)
    case = wl.make_case("hf", B=5, Hq=8, Hkv=2, d=d, P=16, seq_lens=[300, 517, 130, 260, 33], seed=91)
    last = case.offsets[1:] - 1
    prefix = case.slot_mapping.copy()
    prefix[last] = -1
    cache = gpu_cache(case, slots=prefix)
    bad_case, bad_lens = hostile(case)
    S = pz.pz_decode_attn_n_splits(case.max_pages * case.P, 0, split_tokens) if split_tokens else 0
    wsb = pz.pz_decode_attn_workspace_bytes(case.B, case.Hq, case.d, S) if split_tokens else 0
    ws = torch.full((max(wsb, 4) // 4,), float("nan"), dtype=torch.float32, device=DEV)
    out = torch.full((case.B, case.Hq, case.d), float("nan"), dtype=torch.float32, device=DEV)
    sl = torch.from_numpy(bad_lens).to(DEV)
    sinks = torch.from_numpy(case.sinks).to(DEV)
    pz.pz_decode_attn_append(cache, dev_bits(case.k[last]), dev_bits(case.v[last]), dev_bits(case.q),
                             torch.from_numpy(bad_case.block_table).to(DEV), case.max_pages, sl, case.B, case.Hq,
                             sinks, case.sm_scale, case.k_scale, case.v_scale, 0, split_tokens, S,
                             ws if split_tokens else None, wsb, out)
    if split_tokens:
        pz.pz_decode_attn_splitk_reduce(ws, wsb, case.B, case.Hq, case.d, S, sl, 0, split_tokens, sinks,
                                        case.v_scale, out)
    torch.cuda.synchronize()
    # expected cache: the prefix plus the newest tokens of the sequences with valid inputs (0 and 4)
    placed = prefix.copy()
    placed[last[[0, 4]]] = case.slot_mapping[last[[0, 4]]]
    ok, ov = oracle.new_cache(case.num_pages * case.P, case.Hkv, case.d, fill=0xAA)
    oracle.kv_append(ok, ov, case.k, case.v, placed, case.k_scale, case.v_scale)
    gk, gv = to_oracle_layout(cache)
    assert np.array_equal(gk, ok) and np.array_equal(gv, ov)
    kc, vc = oracle_cache(case)
    want = oracle.decode_attn(kc, vc, case.P, case.q, case.block_table, case.seq_lens, sinks=case.sinks,
                              sm_scale=case.sm_scale, k_scale=case.k_scale, v_scale=case.v_scale, window=0, nthreads=8)
    got = out.cpu().numpy()
    for b in (0, 4):
        assert rel_err(got[b], want[b]) <= TOL, b
    assert np.all(got[3] == 0.0)


@pytest.mark.parametrize("form", ["tile", "token"])
@pytest.mark.parametrize("rope,d", [(False, 64), (True, 64), (False, 128)])
def test_append_skips_slots_outside_the_cache(form, rope, d, launch_override):
    launch_override("append_form", pz.APPEND_FORM_TOKEN if form == "token" else pz.APPEND_FORM_TILE)
    Hkv, P, T, num_pages = 2, 16, 150, 12
    rng = np.random.default_rng(5)
    k = wl.bf16_bits(rng.standard_normal((T, Hkv, d)).astype(np.float32))
    v = wl.bf16_bits(rng.standard_normal((T, Hkv, d)).astype(np.float32))
    slots = rng.permutation(num_pages * P)[:T].astype(np.int64)
    outside = np.array([num_pages * P, num_pages * P + 3, 2 ** 40, 2 ** 62, -1, -2 ** 62], dtype=np.int64)
    slots[::9] = outside[np.arange(len(slots[::9])) % len(outside)]
    kept = np.where((slots >= 0) & (slots < num_pages * P), slots, -1)
    cache = pz.PagedCache.allocate(num_pages, P, Hkv, d, pz.KV_FP8, DEV, fill=0xAA)
    sm = torch.from_numpy(slots).to(DEV)
    ok, ov = oracle.new_cache(num_pages * P, Hkv, d, fill=0xAA)
    if rope:
        n_pos, Hq = 64, 4
        cos, sin = pz.pz_rope_yarn_table(pz.YarnParams(factor=32.0), d, n_pos)
        pos = rng.integers(0, n_pos, size=T).astype(np.int32)
        q = wl.bf16_bits(rng.standard_normal((T, Hq, d)).astype(np.float32))
        q_dev = dev_bits(q)
        pz.pz_rope_kv_append_fp8(cache, q_dev, q_dev, dev_bits(k), dev_bits(v), torch.from_numpy(pos).to(DEV),
                                 torch.from_numpy(cos).to(DEV), torch.from_numpy(sin).to(DEV), sm, T, Hq, 0.02, 0.03)
        oq = oracle.rope_kv_append(ok, ov, q, k, v, pos, cos, sin, kept, 0.02, 0.03)
        torch.cuda.synchronize()
        assert np.array_equal(q_dev.cpu().numpy().view(np.uint16), oq)     # every query row is rotated
    else:
        pz.pz_kv_append_fp8(cache, dev_bits(k), dev_bits(v), sm, T, 0.02, 0.03)
        oracle.kv_append(ok, ov, k, v, kept, 0.02, 0.03)
    torch.cuda.synchronize()
    gk, gv = to_oracle_layout(cache)
    assert np.array_equal(gk, ok) and np.array_equal(gv, ov)


def test_prefill_with_hostile_tables_and_lengths():
    case = wl.make_case("hp", B=5, Hq=8, Hkv=2, d=64, P=16, seq_lens=[300, 517, 130, 260, 97], seed=93)
    cache = gpu_cache(case)
    kc, vc = oracle_cache(case)
    n_new = [40, 100, 30, 20, 97]
    q_start = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
    T = int(q_start[-1])
    rng = np.random.default_rng(94)
    q = wl.bf16_bits(rng.standard_normal((T, case.Hq, case.d)).astype(np.float32))
    want = oracle.prefill_attn(kc, vc, case.P, q, q_start, case.block_table, case.seq_lens, case.sinks, case.sm_scale,
                               case.k_scale, case.v_scale, 0, accum="f64", nthreads=8)
    bad_case, bad_lens = hostile(case)
    out = torch.full((T, case.Hq, case.d), float("nan"), dtype=torch.float32, device=DEV)
    pz.pz_prefill_attn(cache, dev_bits(q), torch.from_numpy(q_start).to(DEV), torch.from_numpy(bad_case.block_table).to(DEV),
                       case.max_pages, torch.from_numpy(bad_lens).to(DEV), case.B, case.Hq, max(n_new),
                       torch.from_numpy(case.sinks).to(DEV), case.sm_scale, case.k_scale, case.v_scale, 0, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for b in (0, 4):
        rows = slice(q_start[b], q_start[b + 1])
        assert rel_err(got[rows], want[rows]) <= TOL, b
