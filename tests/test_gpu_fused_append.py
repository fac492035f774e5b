"""pz_decode_attn_append (the newest token's quantise-and-append fused into the attention launch)
against the two separate calls and against the oracle.  The cache bytes are the same bit for bit.  The
outputs are bit-identical when the call appends by a launch of its own first; when the append runs inside
the attention launch the newest position is folded into the online softmax last, as a step of its own,
instead of together with the other positions of its 64-position step, so the same sums are rounded in
another order: each weight enters as two truncated bf16 terms (2^-16 relative, one-sided) against a
reference maximum that may differ between the two orders, plus fp32 roundings of the rescaling -- the two
outputs agree to 1e-4 of the output RMS (measured: a few 1e-5), and each meets the bar against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_11937_amd as pz
import workloads as wl
from gpu_helpers import DEV, dev_bits, gpu_cache, to_oracle_layout
from helpers import oracle_cache, rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-3
REGROUP = 1e-4         # fused-in-kernel against append-then-attend: rounding order of the online softmax only


def same_outputs(out_a, out_b, way):
    if way == "own_launch":
        return torch.equal(out_a, out_b)
    a, b = out_a.cpu().numpy(), out_b.cpu().numpy()
    return not np.any(np.isnan(b)) and rel_err(b, a) <= REGROUP

GEOMETRIES = {
    "p64_mixed": dict(B=5, Hq=16, Hkv=2, d=64, P=64, seq_lens=[1500, 64, 65, 1, 129]),
    "p16_g4": dict(B=4, Hq=8, Hkv=2, d=64, P=16, seq_lens=[100, 37, 16, 17]),
    "p32_g1": dict(B=3, Hq=2, Hkv=2, d=64, P=32, seq_lens=[33, 300, 2]),
    "gpt_oss_heads": dict(B=2, Hq=64, Hkv=8, d=64, P=64, seq_lens=[2500, 640]),
    "window": dict(B=4, Hq=16, Hkv=2, d=64, P=64, seq_lens=[1000, 128, 129, 50], window=128),
    "window_unaligned": dict(B=3, Hq=16, Hkv=2, d=64, P=16, seq_lens=[1000, 333, 20], window=300),
    "g16_two_virtual_heads": dict(B=3, Hq=32, Hkv=2, d=64, P=64, seq_lens=[700, 64, 1300]),
    "window128_single_pass": dict(B=6, Hq=16, Hkv=2, d=64, P=64, seq_lens=[1000, 128, 129, 1, 65, 193], window=128),
    "window20_p16_single_pass": dict(B=4, Hq=8, Hkv=2, d=64, P=16, seq_lens=[100, 37, 16, 17], window=20),
    "batch_70_hkv8": dict(B=70, Hq=8, Hkv=8, d=64, P=16, seq_lens=[1 + (37 * i) % 150 for i in range(70)]),
    "g32_four_virtual_heads": dict(B=2, Hq=64, Hkv=2, d=64, P=64, seq_lens=[900, 65]),
    "g9_uneven_parts": dict(B=3, Hq=18, Hkv=2, d=64, P=64, seq_lens=[700, 64, 130]),
    "g33_empty_part": dict(B=2, Hq=33, Hkv=1, d=64, P=16, seq_lens=[200, 17]),
}


def run_pair(case, split_tokens, dtype=pz.KV_FP8):
    """(out, cache) by append + attention, and by the fused call, from the same prefix cache."""
    last = case.offsets[1:] - 1
    slots_prefix = case.slot_mapping.copy()
    slots_prefix[last] = -1
    k_new, v_new = dev_bits(case.k[last]), dev_bits(case.v[last])
    q = dev_bits(case.q)
    bt = torch.from_numpy(case.block_table).to(DEV)
    sl = torch.from_numpy(case.seq_lens).to(DEV)
    sinks = torch.from_numpy(case.sinks).to(DEV)
    ks, vs = (case.k_scale, case.v_scale) if dtype == pz.KV_FP8 else (1.0, 1.0)
    S = pz.pz_decode_attn_n_splits(int(case.seq_lens.max()), case.window, split_tokens) if split_tokens else 0
    wsb = pz.pz_decode_attn_workspace_bytes(case.B, case.Hq, case.d, S) if split_tokens else 0
    res = []
    for fused in (False, True):
        cache = gpu_cache(case, dtype=dtype, slots=slots_prefix, k_scale=ks, v_scale=vs)
        ws = torch.full((max(wsb, 4) // 4,), float("nan"), dtype=torch.float32, device=DEV)
        out = torch.full((case.B, case.Hq, case.d), float("nan"), dtype=torch.float32, device=DEV)
        args = (q, bt, case.max_pages, sl, case.B, case.Hq, sinks, case.sm_scale, ks, vs, case.window, split_tokens, S,
                ws if split_tokens else None, wsb, out)
        if fused:
            pz.pz_decode_attn_append(cache, k_new, v_new, *args)
        else:
            pz.pz_kv_append_fp8(cache, k_new, v_new, torch.from_numpy(case.slot_mapping[last]).to(DEV), case.B, ks, vs)
            pz.pz_decode_attn(cache, *args)
        if split_tokens:
            pz.pz_decode_attn_splitk_reduce(ws, wsb, case.B, case.Hq, case.d, S, sl, case.window, split_tokens, sinks,
                                            vs, out)
        torch.cuda.synchronize()
        res.append((out, cache))
    return res


@pytest.fixture(params=["in_kernel", "own_launch"])
def fused_way(request, launch_override):
    """pz_decode_attn_append writes the token inside the attention launch (single-pass calls) or by a launch of
    its own first (split-K calls); force each way for every call."""
    launch_override("append_fused", 1 if request.param == "in_kernel" else 0)
    return request.param


@pytest.mark.parametrize("name", list(GEOMETRIES))
@pytest.mark.parametrize("split_tokens", [0, 64, 256])
def test_fused_equals_append_then_attention(name, split_tokens, fused_way):
    case = wl.make_case(name, seed=70 + len(name), **GEOMETRIES[name])
    (out_a, cache_a), (out_b, cache_b) = run_pair(case, split_tokens)
    assert torch.equal(cache_a.k, cache_b.k) and torch.equal(cache_a.v, cache_b.v)     # canary bytes included
    assert same_outputs(out_a, out_b, fused_way)
    kc, vc = oracle_cache(case)
    gk, gv = to_oracle_layout(cache_b)
    assert np.array_equal(gk, kc) and np.array_equal(gv, vc)
    want = oracle.decode_attn(kc, vc, case.P, case.q, case.block_table, case.seq_lens, case.sinks, case.sm_scale,
                              case.k_scale, case.v_scale, case.window, accum="f64", nthreads=8)
    assert rel_err(out_b.cpu().numpy(), want) <= TOL


def test_fused_append_into_a_bf16_cache(fused_way):
    case = wl.make_case("b", B=3, Hq=16, Hkv=2, d=64, P=32, seq_lens=[200, 32, 33], seed=81)
    for split in (0, 128):
        (out_a, cache_a), (out_b, cache_b) = run_pair(case, split, dtype=pz.KV_BF16)
        assert torch.equal(cache_a.k, cache_b.k) and torch.equal(cache_a.v, cache_b.v)
        assert same_outputs(out_a, out_b, fused_way)


@pytest.mark.parametrize("waves,cpg", [(1, 1), (1, 3), (2, 1), (4, 1), (8, 1)])
def test_fused_append_under_every_launch_shape(waves, cpg, launch_override):
    launch_override("append_fused", 1)
    launch_override("attn_waves", waves)
    launch_override("attn_chunks_per_group", cpg)
    case = wl.make_case("s", B=4, Hq=16, Hkv=2, d=64, P=64, seq_lens=[3000, 64, 700, 1], seed=82)
    for split in (0, 256):
        (out_a, cache_a), (out_b, cache_b) = run_pair(case, split)
        assert torch.equal(cache_a.k, cache_b.k) and torch.equal(cache_a.v, cache_b.v)
        assert same_outputs(out_a, out_b, "in_kernel")


def test_a_decode_loop_of_fused_steps_matches_the_oracle(fused_way):
    """Twenty consecutive decode steps through the fused call, the sequences growing across page and
    chunk boundaries; after the last step the cache and the output equal the oracle's."""
    full = wl.make_case("l", B=3, Hq=16, Hkv=2, d=64, P=16, seq_lens=[90, 37, 150], seed=83)
    n_steps = 20
    start = full.seq_lens - n_steps
    keep = np.concatenate([np.arange(full.offsets[b], full.offsets[b] + start[b]) for b in range(full.B)])
    slots0 = np.full_like(full.slot_mapping, -1)
    slots0[keep] = full.slot_mapping[keep]
    cache = gpu_cache(full, slots=slots0)
    bt = torch.from_numpy(full.block_table).to(DEV)
    sinks = torch.from_numpy(full.sinks).to(DEV)
    out = torch.zeros((full.B, full.Hq, full.d), dtype=torch.float32, device=DEV)
    rng = np.random.default_rng(5)
    for t in range(n_steps):
        L = (start + t + 1).astype(np.int32)
        idx = full.offsets[:-1] + start + t
        q = wl.bf16_bits(rng.standard_normal((full.B, full.Hq, full.d)).astype(np.float32))
        pz.pz_decode_attn_append(cache, dev_bits(full.k[idx]), dev_bits(full.v[idx]), dev_bits(q), bt, full.max_pages,
                                 torch.from_numpy(L).to(DEV), full.B, full.Hq, sinks, full.sm_scale, full.k_scale,
                                 full.v_scale, 0, 0, 0, None, 0, out)
    torch.cuda.synchronize()
    kc, vc = oracle_cache(full)
    gk, gv = to_oracle_layout(cache)
    assert np.array_equal(gk, kc) and np.array_equal(gv, vc)
    want = oracle.decode_attn(kc, vc, full.P, q, full.block_table, full.seq_lens, full.sinks, full.sm_scale,
                              full.k_scale, full.v_scale, 0, accum="f64", nthreads=8)
    assert rel_err(out.cpu().numpy(), want) <= TOL
