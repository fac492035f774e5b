"""pz_decode_attn_noalloc (split-K partials in the library's own device array, no workspace argument, no
allocation) against pz_decode_attn + pz_decode_attn_splitk_reduce with a caller-owned workspace: same
kernels, so the outputs must be bit-identical, on two calls in a row, the second smaller than the first
(it finds the first call's partials in the array and must not use them), then a larger one again and a
window layer; and against the oracle within the output tolerance.  Collected last: a failure here must
not hide the tests before it."""
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


def noalloc_attn(case, cache, window, split_tokens, out_dtype=pz.OUT_F32, check=True):
    S = pz.pz_decode_attn_n_splits(int(case.seq_lens.max(initial=0)), window, split_tokens) if split_tokens else 0
    tdt = torch.float32 if out_dtype == pz.OUT_F32 else torch.bfloat16
    out = torch.full((case.B, case.Hq, case.d), float("nan"), dtype=tdt, device=DEV)
    sk = torch.from_numpy(case.sinks).to(DEV)
    st = pz.pz_decode_attn_noalloc(cache, dev_bits(case.q), torch.from_numpy(case.block_table).to(DEV), case.max_pages,
                                   torch.from_numpy(case.seq_lens).to(DEV), case.B, case.Hq, sk, case.sm_scale,
                                   case.k_scale, case.v_scale, window, split_tokens, S, out, out_dtype, check=check)
    torch.cuda.synchronize()
    return st, out.float().cpu().numpy()


def test_two_calls_in_a_row_the_second_smaller_match_the_workspace_calls():
    calls = [
        # (name, B, Hq, Hkv, lengths, window, split)
        ("large", 6, 16, 2, [5000, 130, 2900, 64, 0, 4097], 0, 256),
        ("small", 2, 16, 2, [700, 90], 0, 256),
        ("large_again", 5, 16, 2, [3000, 1, 2999, 640, 1500], 0, 128),
        ("window", 4, 8, 8, [2500, 300, 64, 1200], 600, 128),
        ("single_pass", 3, 8, 2, [100, 37, 1], 0, 0),
    ]
    before = torch.cuda.memory_allocated()
    for i, (name, B, Hq, Hkv, lens, window, split) in enumerate(calls):
        case = wl.make_case(name, B=B, Hq=Hq, Hkv=Hkv, d=64, P=64, seq_lens=lens, window=window, seed=300 + i)
        cache = gpu_cache(case)
        st, got = noalloc_attn(case, cache, window, split)
        assert st == 0, name
        ref = gpu_attn(case, cache, window=window, split_tokens=split)
        assert np.array_equal(got, ref), name                      # same kernels, same order of operations
        kc, vc = oracle_cache(case)
        want = oracle.decode_attn(kc, vc, case.P, case.q, case.block_table, case.seq_lens, case.sinks, case.sm_scale,
                                  case.k_scale, case.v_scale, window, accum="f64")
        assert rel_err(got, want) <= TOL, name
        assert np.all(got[np.asarray(lens) == 0] == 0)
        del cache
    assert torch.cuda.memory_allocated() <= before + (1 << 20)      # nothing of the calls stays allocated


def test_bf16_output_and_the_size_limit():
    case = wl.make_case("lim", B=2, Hq=16, Hkv=2, d=64, P=64, seq_lens=[900, 400], seed=310)
    cache = gpu_cache(case)
    st, got = noalloc_attn(case, cache, 0, 128, out_dtype=pz.OUT_BF16)
    ref = gpu_attn(case, cache, split_tokens=128, out_dtype=pz.OUT_BF16)
    assert st == 0 and np.array_equal(got, ref)
    # a call whose partials would not fit the array is refused on the host, before anything is enqueued
    q = dev_bits(case.q)
    bt = torch.from_numpy(case.block_table).to(DEV)
    sl = torch.from_numpy(case.seq_lens).to(DEV)
    out = torch.zeros((case.B, case.Hq, case.d), dtype=torch.float32, device=DEV)
    too_many = pz.NOALLOC_WORKSPACE_BYTES // (case.B * case.Hq * 66 * 4) + 1
    assert pz.pz_decode_attn_workspace_bytes(case.B, case.Hq, 64, too_many) > pz.NOALLOC_WORKSPACE_BYTES
    st = pz.pz_decode_attn_noalloc(cache, q, bt, case.max_pages, sl, case.B, case.Hq, None, case.sm_scale, case.k_scale,
                                   case.v_scale, 0, 64, too_many, out, check=False)
    assert st == -4
    fits = too_many - 1
    st = pz.pz_decode_attn_noalloc(cache, q, bt, case.max_pages, sl, case.B, case.Hq, None, case.sm_scale, case.k_scale,
                                   case.v_scale, 0, 64, fits, out, check=False)
    torch.cuda.synchronize()
    assert st == 0
    ref = gpu_attn(case, cache, split_tokens=64, sinks=None, n_splits=fits)
    assert np.array_equal(out.cpu().numpy(), ref)


def test_recorded_into_a_hip_graph_and_replayed():
    """What the entry point is for: a capture in which nothing may allocate.  The first call on the device is
    made eagerly (it looks up the array's address); the captured call then only enqueues kernels, and every
    replay -- with other calls of the same entry point, on other sizes, between the replays -- gives the eager
    result."""
    case = wl.make_case("cap", B=4, Hq=16, Hkv=2, d=64, P=64, seq_lens=[1500, 64, 700, 129], seed=320)
    other = wl.make_case("cap2", B=2, Hq=16, Hkv=2, d=64, P=64, seq_lens=[300, 2000], seed=321)
    cache, cache2 = gpu_cache(case), gpu_cache(other)
    q, bt = dev_bits(case.q), torch.from_numpy(case.block_table).to(DEV)
    sl, sinks = torch.from_numpy(case.seq_lens).to(DEV), torch.from_numpy(case.sinks).to(DEV)
    split = 256
    S = pz.pz_decode_attn_n_splits(1500, 0, split)
    out = torch.zeros((case.B, case.Hq, case.d), dtype=torch.float32, device=DEV)

    def call():
        pz.pz_decode_attn_noalloc(cache, q, bt, case.max_pages, sl, case.B, case.Hq, sinks, case.sm_scale, case.k_scale,
                                  case.v_scale, 0, split, S, out)

    call()
    torch.cuda.synchronize()
    eager = out.clone()
    assert np.array_equal(eager.cpu().numpy(), gpu_attn(case, cache, split_tokens=split))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            call()
    torch.cuda.current_stream().wait_stream(side)
    for i in range(3):
        out.fill_(float("nan"))
        st, got2 = noalloc_attn(other, cache2, 0, 128)             # leaves other partials in the array
        assert st == 0 and np.array_equal(got2, gpu_attn(other, cache2, split_tokens=128))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), i
