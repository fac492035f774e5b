"""Full-size parity on sampled sequences, in the launch configuration bench.py times.

The configurations are the benchmark's (gpt-oss head geometry, page 64): the inputs are drawn on
the device by workloads.device_layer, the cache is built by pz_kv_append_fp8, and the oracle
recomputes a few whole sequences from the same bf16 K/V (its own quantisation, its own layout)."""
import numpy as np
import pytest
import torch

import bench
import oracle
import paper_2602_11937_amd as pz
import workloads as wl
from helpers import rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-3


def oracle_sequences(layer, seqs, accum):
    """Oracle output rows [len(seqs)][Hq][d] for the listed sequences of a bench Layer."""
    lay = layer.lay
    P = lay.P
    off = np.concatenate([[0], np.cumsum(lay.seq_lens.astype(np.int64))])
    n_pages = [-(-int(lay.seq_lens[b]) // P) for b in seqs]
    bt = np.full((len(seqs), max(n_pages)), -1, dtype=np.int32)
    at = 0
    for i in range(len(seqs)):
        bt[i, :n_pages[i]] = np.arange(at, at + n_pages[i])
        at += n_pages[i]
    kc, vc = oracle.new_cache(at * P, lay.Hkv, lay.d, oracle.KV_FP8)
    for i, b in enumerate(seqs):
        L = int(lay.seq_lens[b])
        kb = lay.k_ctx[off[b]:off[b + 1]].view(torch.int16).cpu().numpy().view(np.uint16)
        vb = lay.v_ctx[off[b]:off[b + 1]].view(torch.int16).cpu().numpy().view(np.uint16)
        j = np.arange(L, dtype=np.int64)
        oracle.kv_append(kc, vc, kb, vb, bt[i, j // P].astype(np.int64) * P + j % P, lay.k_scale, lay.v_scale)
        # the GPU cache bytes of this sequence, read through the block table, are the oracle's bytes
        pages = torch.from_numpy(lay.block_table_host[b, :n_pages[i]].astype(np.int64)).cuda()
        gk = layer.cache.k[pages].permute(0, 2, 1, 3).reshape(-1, lay.Hkv, lay.d)[:L].cpu().numpy()
        gv = layer.cache.v[pages].permute(0, 3, 1, 2).reshape(-1, lay.Hkv, lay.d)[:L].cpu().numpy()
        first = int(bt[i, 0]) * P
        assert np.array_equal(gk, kc[first:first + L]) and np.array_equal(gv, vc[first:first + L])
    q = lay.q[seqs].view(torch.int16).cpu().numpy().view(np.uint16)
    return oracle.decode_attn(kc, vc, P, q, bt, lay.seq_lens[seqs], lay.sinks.cpu().numpy(), lay.sm_scale,
                              lay.k_scale, lay.v_scale, layer.window, accum=accum, nthreads=16)


@pytest.mark.parametrize("name,seqs", [("cfg3", [0, 9]), ("cfg2", [3, 40, 63]), ("cfg4_w128", [0, 100, 255]),
                                       ("cfg4_w8192", [0, 100, 255])])
def test_bench_configuration_against_oracle_on_sampled_sequences(name, seqs):
    spec = bench.WORKLOADS[name]
    layer = bench.Layer(pz, wl, torch, spec, seed=spec["seed"], kv_dtype=pz.KV_FP8, keep_context=True)
    layer.out.fill_(float("nan"))
    layer.step()
    torch.cuda.synchronize()
    out = layer.out.cpu().numpy()
    assert not np.any(np.isnan(out))
    # properties that hold at any size: heads of a group differ, rows are bounded by |V|max * v_scale
    assert np.max(np.abs(out)) <= 448.0 * layer.v_scale * (1 + 1e-5)
    got = out[seqs]
    e32 = rel_err(got, oracle_sequences(layer, seqs, "f32"))
    e64 = rel_err(got, oracle_sequences(layer, seqs, "f64"))
    print("%s: sampled sequences %s: err vs f32 oracle %.2e, vs f64 oracle %.2e" % (name, seqs, e32, e64))
    assert e32 <= TOL and e64 <= TOL
    layer.lay.k_ctx = layer.lay.v_ctx = None
    del layer
    torch.cuda.empty_cache()
