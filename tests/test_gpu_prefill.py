"""GPU parity of multi-token (prefill / chunked-prefill) attention against the oracle's definition."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_11937_amd as pz
import workloads as wl
from gpu_helpers import DEV, dev_bits, gpu_attn, gpu_cache
from helpers import oracle_cache, rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-3


def gpu_prefill(case, cache, q, n_new, window, out_dtype=pz.OUT_F32):
    q_start = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
    T = int(q_start[-1])
    tdt = torch.float32 if out_dtype == pz.OUT_F32 else torch.bfloat16
    out = torch.full((T, case.Hq, case.d), float("nan"), dtype=tdt, device=DEV)
    pz.pz_prefill_attn(cache, dev_bits(q), torch.from_numpy(q_start).to(DEV), torch.from_numpy(case.block_table).to(DEV),
                       case.max_pages, torch.from_numpy(case.seq_lens).to(DEV), case.B, case.Hq, int(max(n_new)),
                       torch.from_numpy(case.sinks).to(DEV) if case.sinks is not None else None, case.sm_scale,
                       case.k_scale, case.v_scale, window, out, out_dtype)
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), q_start


@pytest.mark.parametrize("kw,n_new", [
    (dict(B=2, Hq=8, Hkv=2, d=64, P=16, seq_lens=[100, 37]), [100, 37]),        # whole prompt, page 16, G 4
    (dict(B=3, Hq=16, Hkv=2, d=64, P=64, seq_lens=[1000, 65, 300]), [1, 5, 300]),  # chunked: 1, odd, all
    (dict(B=2, Hq=64, Hkv=8, d=64, P=64, seq_lens=[700, 130]), [130, 130]),     # gpt-oss heads
    (dict(B=2, Hq=2, Hkv=2, d=64, P=32, seq_lens=[90, 33]), [7, 33]),           # G 1
    (dict(B=3, Hq=16, Hkv=2, d=64, P=64, seq_lens=[500, 64, 1], sinks=False), [64, 0, 1]),   # a sequence without queries
    (dict(B=2, Hq=24, Hkv=2, d=64, P=64, seq_lens=[200, 77]), [9, 77]),         # G 12: two virtual heads per KV head
    (dict(B=2, Hq=32, Hkv=1, d=64, P=64, seq_lens=[150, 77]), [40, 77]),        # G 32: four
    (dict(B=2, Hq=18, Hkv=2, d=64, P=64, seq_lens=[150, 77]), [40, 77]),        # G 9: parts of 5 and 4
    (dict(B=1, Hq=33, Hkv=1, d=64, P=32, seq_lens=[130]), [130]),                # G 33: seven parts and an empty one
])
@pytest.mark.parametrize("window", [0, 128, 50])
def test_prefill_matches_oracle(kw, n_new, window):
    case = wl.make_case("pf", seed=len(n_new) + window, **kw)
    cache = gpu_cache(case, fill=0x7F)
    kc, vc = oracle_cache(case)
    rng = np.random.default_rng(window)
    T = int(np.sum(n_new))
    q = wl.bf16_bits(rng.standard_normal((T, case.Hq, case.d)).astype(np.float32))
    got, q_start = gpu_prefill(case, cache, q, n_new, window)
    want = oracle.prefill_attn(kc, vc, case.P, q, q_start, case.block_table, case.seq_lens, case.sinks,
                               case.sm_scale, case.k_scale, case.v_scale, window, accum="f64", nthreads=8)
    assert not np.any(np.isnan(got)) and rel_err(got, want) <= TOL


def test_prefill_of_one_token_is_the_decode_call_and_bf16_out():
    case = wl.make_case("pd", B=3, Hq=16, Hkv=2, d=64, P=64, seq_lens=[400, 64, 129], seed=3)
    cache = gpu_cache(case)
    dec = gpu_attn(case, cache)
    got, _ = gpu_prefill(case, cache, case.q, [1, 1, 1], 0)
    assert rel_err(got, dec) < 1e-4
    b16, _ = gpu_prefill(case, cache, case.q, [1, 1, 1], 0, out_dtype=pz.OUT_BF16)
    assert np.array_equal(b16, torch.from_numpy(got).to(torch.bfloat16).float().numpy())


def test_chunked_prefill_equals_one_shot():
    """Feeding a prompt in chunks (append chunk, attend, append next chunk ...) gives the rows of the one-shot call."""
    case = wl.make_case("pc", B=1, Hq=16, Hkv=2, d=64, P=64, seq_lens=[333], window=100, seed=4)
    rng = np.random.default_rng(4)
    q = wl.bf16_bits(rng.standard_normal((333, case.Hq, case.d)).astype(np.float32))
    full_cache = gpu_cache(case)
    want, _ = gpu_prefill(case, full_cache, q, [333], 100)
    cache = pz.PagedCache.allocate(case.num_pages, case.P, case.Hkv, case.d, pz.KV_FP8, DEV, fill=0x7F)
    done, rows = 0, []
    for n in (64, 1, 200, 68):
        sl = torch.from_numpy(case.slot_mapping[done:done + n]).to(DEV)
        pz.pz_kv_append_fp8(cache, dev_bits(case.k[done:done + n]), dev_bits(case.v[done:done + n]), sl, n,
                            case.k_scale, case.v_scale)
        done += n
        part = wl.Case(**{**case.__dict__, "seq_lens": np.array([done], dtype=np.int32)})
        got, _ = gpu_prefill(part, cache, q[done - n:done], [n], 100)
        rows.append(got)
    assert rel_err(np.concatenate(rows), want) < 1e-5


@pytest.mark.parametrize("window", [0, 700])
@pytest.mark.parametrize("kv", ["fp8", "bf16"])
def test_long_prompt_on_both_cache_dtypes(window, kv):
    """Hundreds of query tokens per sequence (many column tiles, a ragged last one), a window that starts
    inside the prompt, and the BF16 cache variant of the same kernel."""
    case = wl.make_case("pl", B=2, Hq=16, Hkv=2, d=64, P=64, seq_lens=[1500, 333], seed=21)
    if kv == "bf16":
        case = wl.Case(**{**case.__dict__, "k_scale": 1.0, "v_scale": 1.0})
    n_new = [517, 333]
    cache = gpu_cache(case, dtype=pz.KV_BF16 if kv == "bf16" else pz.KV_FP8)
    kc, vc = oracle_cache(case, oracle.KV_BF16 if kv == "bf16" else oracle.KV_FP8)
    q = wl.bf16_bits(np.random.default_rng(5).standard_normal((sum(n_new), case.Hq, case.d)).astype(np.float32))
    got, q_start = gpu_prefill(case, cache, q, n_new, window)
    want = oracle.prefill_attn(kc, vc, case.P, q, q_start, case.block_table, case.seq_lens, case.sinks,
                               case.sm_scale, case.k_scale, case.v_scale, window, accum="f64", nthreads=8)
    assert not np.any(np.isnan(got)) and rel_err(got, want) <= TOL
