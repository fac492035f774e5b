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


def oracle_sequences(layer, seqs):
    """Oracle output rows [len(seqs)][Hq][d] (fp32 and fp64 arithmetic) for sequences of a bench Layer."""
    lay = layer.lay
    P = lay.P
    kc, vc, bt, q, new_k, new_v, new_slots = bench.oracle_sample(oracle, torch, layer, seqs)
    oracle.kv_append(kc, vc, new_k, new_v, new_slots, lay.k_scale, lay.v_scale)
    for i, b in enumerate(seqs):
        # the GPU cache bytes of the resident positions, read through the block table, are the oracle's
        L, fp = int(lay.seq_lens[b]), int(lay.first_pos[b])
        p0, p1 = fp // P, -(-L // P)
        pages = torch.from_numpy(lay.block_table_host[b, p0:p1].astype(np.int64)).cuda()
        gk = layer.cache.k[pages].permute(0, 2, 1, 3).reshape(-1, lay.Hkv, lay.d)[:L - fp].cpu().numpy()
        gv = layer.cache.v[pages].permute(0, 3, 1, 2).reshape(-1, lay.Hkv, lay.d)[:L - fp].cpu().numpy()
        first = int(bt[i, p0]) * P
        assert np.array_equal(gk, kc[first:first + L - fp]) and np.array_equal(gv, vc[first:first + L - fp])
    sinks = lay.sinks.cpu().numpy()
    return [oracle.decode_attn(kc, vc, P, q, bt, lay.seq_lens[seqs], sinks, lay.sm_scale, lay.k_scale,
                               lay.v_scale, layer.window, accum=a, nthreads=16) for a in ("f32", "f64")]


@pytest.mark.parametrize("name,seqs", [("cfg3", [0, 9]), ("cfg2", [3, 40, 63]), ("cfg4_w128", [0, 100, 255]),
                                       ("cfg4_w8192", [0, 100, 255]), ("cfg5_w128", [0, 31]),
                                       ("cfg5_w8192", [0, 17, 31]), ("cfg5_full", [5, 31])])
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
    want32, want64 = oracle_sequences(layer, seqs)
    e32, e64 = rel_err(got, want32), rel_err(got, want64)
    print("%s: sampled sequences %s: err vs f32 oracle %.2e, vs f64 oracle %.2e" % (name, seqs, e32, e64))
    assert e32 <= TOL and e64 <= TOL
    layer.lay.k_ctx = layer.lay.v_ctx = None
    del layer
    torch.cuda.empty_cache()
