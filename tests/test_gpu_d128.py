"""GPU parity of the 128-channel-head form (quantise-and-append, decode attention single pass and split-K,
merge, the fused-append entry, the entry point that allocates nothing) against the oracle, which is written
for any head dimension.  Cache bytes bit-exact, outputs within 2e-3 of the output RMS."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_11937_amd as pz
import workloads as wl
from gpu_helpers import DEV, dev_bits, gpu_attn, gpu_cache, to_oracle_layout
from helpers import check_workspace_rows, oracle_cache, rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-3

GEOMETRIES = {
    "p64_mixed": dict(B=5, Hq=16, Hkv=2, P=64, seq_lens=[1500, 64, 65, 1, 129]),
    "p16_g4": dict(B=4, Hq=8, Hkv=2, P=16, seq_lens=[100, 37, 16, 17]),
    "p32_g1": dict(B=3, Hq=2, Hkv=2, P=32, seq_lens=[33, 300, 2]),
    "eight_kv_heads": dict(B=2, Hq=64, Hkv=8, P=64, seq_lens=[2500, 640]),
    "window": dict(B=4, Hq=16, Hkv=2, P=64, seq_lens=[1000, 128, 129, 50], window=128),
    "window_unaligned": dict(B=3, Hq=16, Hkv=2, P=16, seq_lens=[1000, 333, 20], window=300),
    "g16_two_virtual_heads": dict(B=3, Hq=32, Hkv=2, P=64, seq_lens=[700, 64, 1300]),
    "g9_uneven_parts": dict(B=3, Hq=18, Hkv=2, P=64, seq_lens=[700, 64, 130]),
    "empty_sequence": dict(B=3, Hq=8, Hkv=2, P=64, seq_lens=[0, 200, 64]),
    "long_with_outliers": dict(B=2, Hq=16, Hkv=2, P=64, seq_lens=[9000, 4100], outlier_frac=0.02),
}


def oracle_out(case, kc, vc, window=None, k_scale=None, v_scale=None, sinks="case"):
    return oracle.decode_attn(kc, vc, case.P, case.q, case.block_table, case.seq_lens,
                              case.sinks if isinstance(sinks, str) else sinks, case.sm_scale,
                              case.k_scale if k_scale is None else k_scale, case.v_scale if v_scale is None else v_scale,
                              case.window if window is None else window, accum="f64", nthreads=8)


@pytest.mark.parametrize("name", list(GEOMETRIES))
def test_append_and_attention_match_the_oracle(name, launch_override):
    case = wl.make_case(name, d=128, seed=400 + len(name), **GEOMETRIES[name])
    kc, vc = oracle_cache(case)
    want = oracle_out(case, kc, vc)
    for form in (pz.APPEND_FORM_TILE, pz.APPEND_FORM_TOKEN):
        launch_override("append_form", form)
        cache = gpu_cache(case)
        gk, gv = to_oracle_layout(cache)
        assert np.array_equal(gk, kc) and np.array_equal(gv, vc), form       # canary bytes included
    for split in (0, 64, 256, 1024):
        got = gpu_attn(case, cache, split_tokens=split)
        assert not np.any(np.isnan(got)) and rel_err(got, want) <= TOL, split
    got = gpu_attn(case, cache, sinks=None)
    assert rel_err(got, oracle_out(case, kc, vc, sinks=None)) <= TOL
    b16 = gpu_attn(case, cache, out_dtype=pz.OUT_BF16)
    f32 = gpu_attn(case, cache)
    assert np.array_equal(b16, torch.from_numpy(f32).to(torch.bfloat16).float().numpy())


@pytest.mark.parametrize("cpg", [1, 3, 8])
def test_workspace_rows_and_chunk_groups(cpg, launch_override):
    """A one-wave workgroup walks `cpg` chunks and leaves one partial in the row of the first; the rows against
    the oracle's chunked definition, and the merged output."""
    launch_override("attn_chunks_per_group", cpg)
    case = wl.make_case("ws", B=3, Hq=16, Hkv=2, d=128, P=64, seq_lens=[1000, 130, 64], seed=418)
    cache = gpu_cache(case)
    kc, vc = oracle_cache(case)
    for window in (0, 300):
        got, acc, ml = gpu_attn(case, cache, window=window, split_tokens=128, return_ws=True)
        S = acc.shape[2]
        oacc, oml = oracle.decode_attn_partials(kc, vc, case.P, case.q, case.block_table, case.seq_lens, case.sm_scale,
                                                case.k_scale, window, 128, S, accum="f64")
        assert check_workspace_rows(acc, ml, oacc, oml, TOL, lse_tol=1.5e-4) >= case.B * case.Hq
        assert rel_err(got, oracle_out(case, kc, vc, window=window)) <= TOL


def test_bf16_cache():
    case = wl.make_case("b", B=3, Hq=16, Hkv=2, d=128, P=32, seq_lens=[700, 32, 130], seed=419)
    cache = gpu_cache(case, dtype=pz.KV_BF16)
    kb, vb = oracle_cache(case, oracle.KV_BF16)
    gk, gv = to_oracle_layout(cache)
    assert np.array_equal(gk, kb) and np.array_equal(gv, vb)
    for split, window in ((0, 0), (128, 0), (0, 100), (64, 100)):
        want = oracle_out(case, kb, vb, window=window, k_scale=1.0, v_scale=1.0)
        got = gpu_attn(case, cache, k_scale=1.0, v_scale=1.0, split_tokens=split, window=window)
        assert rel_err(got, want) <= TOL


@pytest.mark.parametrize("split", [0, 256])
def test_fused_append_entry_and_noalloc_entry(split):
    case = wl.make_case("f", B=4, Hq=16, Hkv=2, d=128, P=64, seq_lens=[1500, 64, 65, 1], seed=420)
    kc, vc = oracle_cache(case)
    want = oracle_out(case, kc, vc)
    last = case.offsets[1:] - 1
    prefix = case.slot_mapping.copy()
    prefix[last] = -1
    cache = gpu_cache(case, slots=prefix)
    q, bt = dev_bits(case.q), torch.from_numpy(case.block_table).to(DEV)
    sl, sinks = torch.from_numpy(case.seq_lens).to(DEV), torch.from_numpy(case.sinks).to(DEV)
    S = pz.pz_decode_attn_n_splits(int(case.seq_lens.max()), 0, split) if split else 0
    wsb = pz.pz_decode_attn_workspace_bytes(case.B, case.Hq, case.d, S) if split else 0
    ws = torch.full((max(wsb, 4) // 4,), float("nan"), dtype=torch.float32, device=DEV)
    out = torch.full((case.B, case.Hq, case.d), float("nan"), dtype=torch.float32, device=DEV)
    pz.pz_decode_attn_append(cache, dev_bits(case.k[last]), dev_bits(case.v[last]), q, bt, case.max_pages, sl, case.B,
                             case.Hq, sinks, case.sm_scale, case.k_scale, case.v_scale, 0, split, S,
                             ws if split else None, wsb, out)
    if split:
        pz.pz_decode_attn_splitk_reduce(ws, wsb, case.B, case.Hq, case.d, S, sl, 0, split, sinks, case.v_scale, out)
    torch.cuda.synchronize()
    gk, gv = to_oracle_layout(cache)
    assert np.array_equal(gk, kc) and np.array_equal(gv, vc)
    assert rel_err(out.cpu().numpy(), want) <= TOL
    out2 = torch.full_like(out, float("nan"))
    pz.pz_decode_attn_noalloc(cache, q, bt, case.max_pages, sl, case.B, case.Hq, sinks, case.sm_scale, case.k_scale,
                              case.v_scale, 0, split, S, out2)
    torch.cuda.synchronize()
    assert torch.equal(out2, out)


def test_entry_points_for_64_channel_heads_refuse_128():
    case = wl.make_case("r", B=1, Hq=8, Hkv=2, d=128, P=64, seq_lens=[70], seed=421)
    cache = gpu_cache(case)
    q = dev_bits(case.q)
    out = torch.zeros((1, case.Hq, case.d), dtype=torch.float32, device=DEV)
    st = pz.pz_prefill_attn(cache, q, torch.tensor([0, 1], dtype=torch.int32, device=DEV),
                            torch.from_numpy(case.block_table).to(DEV), case.max_pages,
                            torch.from_numpy(case.seq_lens).to(DEV), 1, case.Hq, 1, None, case.sm_scale, case.k_scale,
                            case.v_scale, 0, out, check=False)
    assert st == -3
