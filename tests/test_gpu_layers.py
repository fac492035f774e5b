"""GPU parity of the heterogeneous 36-layer decode step (the per-layer loop of
paper_2602_11937_amd.decode_step) against the oracle, layer by layer.

The layer pattern is the paper's: layers alternate window 128 and global attention, and 8 of the 18
global layers are turned into window 8192 (Section 2, "Window attention for long-context inference");
every layer has its own K and V scale (Section 3, "KV Quantization").  Here at reduced batch and context
so that the oracle covers every sequence of every layer: batch 3, contexts up to 8700 (so that window
8192 differs from full attention for the longest sequence), independent K/V data and clearly different
magnitudes -- hence scales -- per layer, window layers holding only the pages their window can touch
(block-table entries before it are -1), one split-K workspace shared by all layers.  Compared for every
layer: the cache bytes after the step (bit-exact; the step appends the newest token of each sequence)
and the output (2e-3 of its RMS), for the FP8 cache and for the BF16 cache, with the append as a call of
its own and fused into the attention call."""
import functools

import numpy as np
import pytest
import torch

import oracle
import paper_2602_11937_amd as pz
import workloads as wl
from gpu_helpers import DEV, dev_bits, to_oracle_layout
from helpers import paper_values, rel_err
from paper_2602_11937_amd.decode_step import DecodeLayer, DecodeStep, LayerInputs

pytestmark = pytest.mark.gpu
TOL = 2e-3
B, HQ, HKV, D, P = 3, 64, 8, 64, 64
LENS = np.array([8700, 2100, 300], dtype=np.int32)
SPLIT = 1024


@functools.lru_cache(maxsize=None)
def layer_case(i, window):
    """Layer i's own inputs (both cache dtypes use the same)."""
    return wl.make_case("layer%d" % i, B=B, Hq=HQ, Hkv=HKV, d=D, P=P, seq_lens=LENS, window=window, seed=500 + i,
                        k_gain=0.5 + 0.25 * (i % 7), v_gain=2.0 ** ((i % 5) - 2))


def build_layer(i, window, kv_dtype):
    """Inputs, device cache (all but the newest token of each sequence appended), oracle cache (everything
    appended by the oracle) of layer i."""
    case = layer_case(i, window)
    L = LENS.astype(np.int64)
    # a window layer keeps the pages of its last window + 64 positions only
    first_pos = (np.maximum(L - (window + 64), 0) // P) * P if window > 0 else np.zeros(B, dtype=np.int64)
    num_pages, bt, slots = wl.paged_tables(np.random.default_rng(900 + i), LENS, P, first_pos=first_pos)
    off = case.offsets
    resident = np.concatenate([np.arange(off[b] + first_pos[b], off[b + 1]) for b in range(B)])
    k, v = case.k[resident], case.v[resident]
    ends = np.cumsum(L - first_pos)
    last = ends - 1                                                  # rows of the newest tokens
    odt = oracle.KV_FP8 if kv_dtype == pz.KV_FP8 else oracle.KV_BF16
    k_scale, v_scale = (case.k_scale, case.v_scale) if kv_dtype == pz.KV_FP8 else (1.0, 1.0)
    okc, ovc = oracle.new_cache(num_pages * P, HKV, D, odt)
    oracle.kv_append(okc, ovc, k, v, slots, k_scale, v_scale)
    want = oracle.decode_attn(okc, ovc, P, case.q, bt, LENS, case.sinks, case.sm_scale, k_scale, v_scale, window,
                              accum="f64", nthreads=8)

    def device_side():
        fill = 0xAA if kv_dtype == pz.KV_FP8 else -21846
        cache = pz.PagedCache.allocate(num_pages, P, HKV, D, kv_dtype, DEV, fill=fill)
        prefix = slots.copy()
        prefix[last] = -1                                            # the step itself appends these
        pz.pz_kv_append_fp8(cache, dev_bits(k), dev_bits(v), torch.from_numpy(prefix).to(DEV), len(prefix), k_scale,
                            v_scale)
        layer = DecodeLayer(cache=cache, block_table=torch.from_numpy(bt).to(DEV), max_pages=int(bt.shape[1]),
                            window=window, k_scale=k_scale, v_scale=v_scale, sm_scale=case.sm_scale,
                            sinks=torch.from_numpy(case.sinks).to(DEV), split_tokens=0 if window == 128 else SPLIT)
        x = LayerInputs(q=dev_bits(case.q), k_new=dev_bits(k[last]), v_new=dev_bits(v[last]),
                        new_slots=torch.from_numpy(slots[last]).to(DEV),
                        out=torch.full((B, HQ, D), float("nan"), dtype=torch.float32, device=DEV))
        return layer, x

    return dict(device_side=device_side, okc=okc, ovc=ovc, want=want, k_scale=k_scale, v_scale=v_scale)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("kv", ["fp8", "bf16"])
def test_the_36_layer_step_matches_the_oracle_layer_by_layer(kv):
    kv_dtype = pz.KV_FP8 if kv == "fp8" else pz.KV_BF16
    pv = paper_values()
    pattern = wl.layer_pattern(seed=5)
    assert len(pattern) == pv["parent_attention_layers"] == 36
    assert pattern.count(128) == 36 - pv["parent_full_attention_layers"] == 18
    assert pattern.count(8192) == pv["converted_layers"] == 8 and pattern.count(0) == 10
    assert set(pattern) == {0, pv["parent_window_tokens"], pv["converted_window_tokens"]}
    built = [build_layer(i, w, kv_dtype) for i, w in enumerate(pattern)]
    if kv == "fp8":                                                  # the per-layer scales really differ
        ks = np.array([b["k_scale"] for b in built])
        assert ks.max() / ks.min() > 3 and len(set(np.round(ks, 6))) >= 7
    seq_lens = torch.from_numpy(LENS).to(DEV)
    outs = {}
    for fused in (False, True):
        sides = [b["device_side"]() for b in built]
        step = DecodeStep([l for l, _ in sides], B, HQ, int(LENS.max()), DEV)
        step.workspace.fill_(float("nan"))                           # shared by all layers, rows reused
        step.run([x for _, x in sides], seq_lens, fused=fused)
        torch.cuda.synchronize()
        worst = 0.0
        for i, ((layer, x), b) in enumerate(zip(sides, built)):
            gk, gv = to_oracle_layout(layer.cache)
            assert np.array_equal(gk, b["okc"]) and np.array_equal(gv, b["ovc"]), (i, pattern[i], fused)
            got = x.out.cpu().numpy()
            assert not np.any(np.isnan(got)), (i, pattern[i], fused)
            err = rel_err(got, b["want"])
            assert err <= TOL, (i, pattern[i], fused, err)
            worst = max(worst, err)
        outs[fused] = [x.out.cpu().numpy() for _, x in sides]
        print("36-layer step, %s cache, fused=%s: worst layer error %.2e of output RMS" % (kv, fused, worst))
    for a, c in zip(outs[False], outs[True]):      # the fused form: the same sums in another rounding order
        assert rel_err(c, a) <= 1e-4
