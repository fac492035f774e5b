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
        L = int(lay.seq_lens[b])
        p0, p1 = int(np.argmax(bt[i] >= 0)), -(-L // P)      # the oracle's copy starts at the window's first page
        fp = p0 * P
        assert fp >= int(lay.first_pos[b]) and (layer.window == 0 or fp <= max(L - layer.window, 0))
        pages = torch.from_numpy(lay.block_table_host[b, p0:p1].astype(np.int64)).cuda()
        gk = layer.cache.k[pages].permute(0, 2, 1, 3).reshape(-1, lay.Hkv, lay.d)[:L - fp].cpu().numpy()
        gv = layer.cache.v[pages].permute(0, 3, 1, 2).reshape(-1, lay.Hkv, lay.d)[:L - fp].cpu().numpy()
        first = int(bt[i, p0]) * P
        assert np.array_equal(gk, kc[first:first + L - fp]) and np.array_equal(gv, vc[first:first + L - fp])
    sinks = lay.sinks.cpu().numpy()
    return [oracle.decode_attn(kc, vc, P, q, bt, lay.seq_lens[seqs], sinks, lay.sm_scale, lay.k_scale,
                               lay.v_scale, layer.window, accum=a, nthreads=bench.host_cores()) for a in ("f32", "f64")]


# The whole batch where the oracle finishes it in seconds (cfg3, cfg2), else a run of consecutive sequences plus
# the last one: shares of the balanced partition and chunk groups that cross from one sequence into the next are
# then compared on both sides of the crossing.
@pytest.mark.timeout(600)
@pytest.mark.parametrize("name,seqs", [("cfg3", list(range(16))), ("cfg2", list(range(64))),
                                       ("cfg4_w128", list(range(256))),
                                       ("cfg4_w8192", list(range(64, 128)) + [0, 255]),
                                       ("cfg5_w128", list(range(32))), ("cfg5_w8192", list(range(8, 20)) + [0, 31]),
                                       ("cfg5_full", list(range(4, 12)) + [31])])
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
    print("%s: %d sampled sequences: err vs f32 oracle %.2e, vs f64 oracle %.2e" % (name, len(seqs), e32, e64))
    # The bar is against the oracle in fp64.  Its fp32 variant adds every sequence's weights and weighted values
    # one after the other in fp32: over L terms of one sign that loses up to L * 2^-24 of the sum (3.9e-3 at
    # 65536 positions; measured 3.3e-3 on the worst of cfg3's sixteen sequences, where the fp64 variant and the
    # GPU agree to 1e-4), so against it the bar is widened by exactly that much.
    L_max = int(layer.lay.seq_lens.max()) if layer.window == 0 else min(int(layer.lay.seq_lens.max()), layer.window)
    assert e64 <= TOL and e32 <= TOL + L_max * 2.0 ** -24
    layer.lay.k_ctx = layer.lay.v_ctx = None
    del layer
    torch.cuda.empty_cache()
