"""Input-recipe checks: layer pattern, byte accounting, paging tables (CPU only).

Facts pinned to the paper: the parent alternates window-128 and full-attention layers (18 of
each over 36 layers) and 8 of the 18 full layers become window-8192 layers (Section 2, "Window
attention for long-context inference"); the resulting KV cache is about 40 % smaller at the
64K-input/64K-output scenario (Section 2, "Optimized Scenarios"); FP8 KV doubles the token
capacity of the cache (Section 3, "KV Quantization").
"""
import numpy as np

import workloads as wl
from helpers import paper_values

PV = paper_values()


def test_layer_pattern_counts():
    pat = wl.layer_pattern()
    n_layers, n_full, n_conv = (int(PV[k]) for k in ("parent_attention_layers", "parent_full_attention_layers",
                                                     "converted_layers"))
    w_par, w_conv = int(PV["parent_window_tokens"]), int(PV["converted_window_tokens"])
    assert (n_layers, n_full, n_conv, w_par, w_conv) == (36, 18, 8, 128, 8192)
    assert len(pat) == n_layers
    assert pat.count(w_par) == n_layers - n_full and pat.count(w_conv) == n_conv and pat.count(0) == n_full - n_conv
    assert all(w == 128 for w in pat[0::2]) and all(w in (0, 8192) for w in pat[1::2])
    assert pat == wl.layer_pattern()                          # seeded, reproducible
    parent = wl.layer_pattern(n_converted=0)
    assert parent.count(128) == 18 and parent.count(0) == 18


def test_kv_cache_is_about_forty_percent_smaller():
    L = int(PV["scenario_input_tokens"] + PV["scenario_output_tokens"])
    assert L == 131072
    child = sum(wl.kv_tokens_read([L], w) for w in wl.layer_pattern())
    parent = sum(wl.kv_tokens_read([L], w) for w in wl.layer_pattern(n_converted=0))
    assert child == 10 * L + 8 * 8192 + 18 * 128 and parent == 18 * L + 18 * 128
    assert abs(child / parent - 0.5837) < 1e-3                # 41.6 % smaller: the paper's "40 %"
    assert abs((1 - child / parent) - PV["kv_cache_fraction_saved"]) < 0.03     # the paper rounds to 40 %
    lens = wl.ragged_lengths(5, 32, 1024, 131072)
    r = (sum(wl.kv_tokens_read(lens, w) for w in wl.layer_pattern())
         / sum(wl.kv_tokens_read(lens, w) for w in wl.layer_pattern(n_converted=0)))
    assert 0.55 < r < 0.66


def test_bytes_per_cached_token():
    assert wl.kv_bytes_per_token(8, 64, 1) == 1024 and wl.kv_bytes_per_token(8, 64, 2) == 2048
    assert wl.kv_bytes_per_token(8, 64, 2) == PV["fp8_token_capacity_factor"] * wl.kv_bytes_per_token(8, 64, 1)
    assert wl.kv_tokens_read([100, 5000, 9000], 8192) == 100 + 5000 + 8192
    assert wl.kv_tokens_read([100, 5000, 9000], 0) == 14100


def test_paged_tables_are_a_partial_permutation():
    case = wl.make_case("t", B=4, Hq=8, Hkv=2, d=64, P=16, seq_lens=[100, 37, 1, 16], seed=3)
    used = case.block_table[case.block_table >= 0]
    assert len(used) == len(set(used.tolist())) == 7 + 3 + 1 + 1
    assert used.max() < case.num_pages and case.num_pages == len(used) + 2
    assert len(set(case.slot_mapping.tolist())) == 154
    off = case.offsets
    for b in range(4):
        j = np.arange(int(case.seq_lens[b]))
        want = case.block_table[b, j // 16].astype(np.int64) * 16 + j % 16
        assert np.array_equal(case.slot_mapping[off[b]:off[b + 1]], want)


def test_scales_are_amax_over_448_and_below_one():
    for case in (wl.config1_tiny(), wl.make_case("o", B=2, Hq=8, Hkv=2, d=64, P=16, seq_lens=[64, 64],
                                                 outlier_frac=0.05, seed=1)):
        for bits, s in ((case.k, case.k_scale), (case.v, case.v_scale)):
            amax = np.max(np.abs(wl.bf16_to_f32(bits)))
            assert s == float(np.float32(amax) / np.float32(448)) and 0 < s < 1
    p2 = wl.make_case("p", B=1, Hq=8, Hkv=2, d=64, P=16, seq_lens=[64], pow2_scales=True)
    raw = wl.make_case("p", B=1, Hq=8, Hkv=2, d=64, P=16, seq_lens=[64])
    for s, r in ((p2.k_scale, raw.k_scale), (p2.v_scale, raw.v_scale)):
        assert np.log2(s) == int(np.log2(s)) and r <= s < 2 * r and s <= 1


def test_outlier_channels_raise_the_k_scale():
    a = wl.make_case("a", B=1, Hq=8, Hkv=2, d=64, P=16, seq_lens=[256], seed=9)
    b = wl.make_case("b", B=1, Hq=8, Hkv=2, d=64, P=16, seq_lens=[256], seed=9, outlier_frac=0.05)
    assert len(b.extra["outlier_pairs"]) == 6 and b.k_scale > 5 * a.k_scale


def test_layer_gains_scale_the_calibrated_scales():
    """k_gain / v_gain multiply K / V before the rounding to bf16, so the max-calibrated scales follow them
    (layers of a model differ in activation magnitude); a power-of-two gain scales the values exactly."""
    import workloads as wl
    a = wl.make_case("g", B=2, Hq=8, Hkv=2, d=64, P=16, seq_lens=[40, 9], seed=3)
    b = wl.make_case("g", B=2, Hq=8, Hkv=2, d=64, P=16, seq_lens=[40, 9], seed=3, k_gain=4.0, v_gain=0.25)
    assert np.array_equal(wl.bf16_to_f32(b.k), 4.0 * wl.bf16_to_f32(a.k))
    assert np.array_equal(wl.bf16_to_f32(b.v), 0.25 * wl.bf16_to_f32(a.v))
    assert b.k_scale == 4.0 * a.k_scale and b.v_scale == 0.25 * a.v_scale
    assert np.array_equal(a.q, b.q) and np.array_equal(a.block_table, b.block_table)


def test_decode_step_sizes_one_workspace_for_the_whole_stack():
    """DecodeStep (the per-layer loop) shares one split-K workspace: as large as the hungriest layer needs, with
    every layer's chunk count from the library's own helper; single-pass layers need none."""
    import torch
    import paper_2602_11937_amd as pz
    from paper_2602_11937_amd.decode_step import DecodeLayer, DecodeStep
    cache = pz.PagedCache(k=None, v=None, num_pages=1, page_size=64, n_kv_heads=8, head_dim=64)
    def layer(window, split):
        return DecodeLayer(cache=cache, block_table=None, max_pages=1, window=window, k_scale=1.0, v_scale=1.0,
                           sm_scale=0.125, sinks=None, split_tokens=split)
    layers = [layer(128, 0), layer(8192, 1024), layer(0, 1024), layer(0, 8192)]
    step = DecodeStep(layers, batch=4, n_q_heads=64, max_seq_len=70000, device="cpu")
    assert step.n_splits == [0, 9, 69, 9]
    assert step.ws_bytes == [0] + [pz.pz_decode_attn_workspace_bytes(4, 64, 64, s) for s in (9, 69, 9)]
    assert step.workspace.numel() * 4 == max(step.ws_bytes) and step.workspace.dtype == torch.float32
