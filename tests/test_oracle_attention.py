"""Pins of the oracle's append, attention, split-K partials and merge (CPU only).

Reference points, none of them the oracle itself: a dense float64 numpy/scipy softmax over the
cache decoded by torch.float8_e4m3fn; torch's own float8 rounding for the append; closed forms
for one key, zero queries and equal keys; exactness properties of scaling by two; the rule that
window attention covers the most recent W tokens (paper Section 2, "Window attention for
long-context inference"), so a window at least as long as the context is full attention.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from helpers import dense_reference, oracle_cache, rel_err, torch_decode_e4m3


def small_case(seed=0, **kw):
    args = dict(B=3, Hq=8, Hkv=2, d=64, P=16, seq_lens=[100, 37, 1])
    args.update(kw)
    return wl.make_case("small", seed=seed, **args)


def run(case, kc, vc, **kw):
    a = dict(sinks=case.sinks, sm_scale=case.sm_scale, k_scale=case.k_scale, v_scale=case.v_scale,
             window=case.window)
    a.update(kw)
    return oracle.decode_attn(kc, vc, case.P, case.q, case.block_table, case.seq_lens, **a)


# ---------------------------------------------------------------- append

def test_append_bytes_match_torch_float8_and_leave_other_slots_alone():
    case = small_case(seed=1)
    kc, vc = oracle_cache(case)
    for cache, x, scale in ((kc, case.k, case.k_scale), (vc, case.v, case.v_scale)):
        r = torch.from_numpy(wl.bf16_to_f32(x)) / torch.tensor(scale, dtype=torch.float32)
        want = r.clamp(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert np.array_equal(cache[case.slot_mapping], want)
        untouched = np.ones(cache.shape[0], dtype=bool)
        untouched[case.slot_mapping] = False
        assert untouched.sum() > 0 and np.all(cache[untouched] == 0xAA)


def test_append_skips_negative_slots_and_is_order_independent():
    case = small_case(seed=2)
    kc, vc = oracle_cache(case)
    T = len(case.slot_mapping)
    perm = np.random.default_rng(0).permutation(T)
    k2, v2 = oracle.new_cache(case.num_pages * case.P, case.Hkv, case.d)
    oracle.kv_append(k2, v2, case.k[perm], case.v[perm], case.slot_mapping[perm], case.k_scale, case.v_scale)
    assert np.array_equal(kc, k2) and np.array_equal(vc, v2)
    slots = case.slot_mapping.copy()
    slots[::3] = -1
    k3, v3 = oracle.new_cache(case.num_pages * case.P, case.Hkv, case.d)
    oracle.kv_append(k3, v3, case.k, case.v, slots, case.k_scale, case.v_scale)
    skipped = case.slot_mapping[::3]
    assert np.all(k3[skipped] == 0xAA) and np.all(v3[skipped] == 0xAA)
    kept = slots[slots >= 0]
    assert np.array_equal(k3[kept], kc[kept]) and np.array_equal(v3[kept], vc[kept])


def test_append_saturates_and_bf16_cache_copies():
    case = small_case(seed=3)
    kc, vc = oracle.new_cache(case.num_pages * case.P, case.Hkv, case.d)
    oracle.kv_append(kc, vc, case.k, case.v, case.slot_mapping, case.k_scale / 50, case.v_scale / 50)
    dec = torch_decode_e4m3(kc[case.slot_mapping])
    assert np.max(np.abs(dec)) == 448.0 and not np.any(np.isnan(dec))
    kb, vb = oracle_cache(case, oracle.KV_BF16)
    assert np.array_equal(kb[case.slot_mapping], case.k) and np.array_equal(vb[case.slot_mapping], case.v)


# ---------------------------------------------------------------- attention vs dense float64

@pytest.mark.parametrize("kw", [
    dict(),                                                   # config-1 geometry: GQA 4, P 16
    dict(Hq=2, Hkv=2, seq_lens=[5, 64, 17]),                  # G = 1
    dict(Hq=8, Hkv=1, seq_lens=[33, 100, 16]),                # G = 8
    dict(P=64, seq_lens=[100, 64, 65]),
    dict(window=20),
    dict(window=16, seq_lens=[100, 16, 15]),
    dict(sinks=False),
    dict(outlier_frac=0.05),
    dict(pow2_scales=True),
    dict(unit_scales=True),
])
def test_attention_matches_dense_float64(kw):
    case = small_case(seed=7, **kw)
    kc, vc = oracle_cache(case)
    want = dense_reference(case, kc, vc)
    assert rel_err(run(case, kc, vc, accum="f64"), want) < 1e-6
    assert rel_err(run(case, kc, vc, accum="f32"), want) < 2e-5


def test_config1_tiny_geometry():
    case = wl.config1_tiny()
    assert (case.B, case.Hq, case.Hkv, case.d, case.P) == (2, 8, 2, 64, 16)
    assert list(case.seq_lens) == [100, 37] and case.sm_scale == 0.125 and case.window == 0
    kc, vc = oracle_cache(case)
    assert rel_err(run(case, kc, vc), dense_reference(case, kc, vc)) < 2e-5


def test_bf16_cache_matches_dense_float64():
    case = small_case(seed=8)
    kb, vb = oracle_cache(case, oracle.KV_BF16)
    got = run(case, kb, vb, k_scale=1.0, v_scale=1.0, accum="f64")
    assert rel_err(got, dense_reference(case, kb, vb, k_scale=1.0, v_scale=1.0)) < 1e-6


def test_rows_subset_and_threads():
    case = small_case(seed=9)
    kc, vc = oracle_cache(case)
    full = run(case, kc, vc)
    rows = np.array([1, 9, 23], dtype=np.int32)
    sub = run(case, kc, vc, rows=rows, nthreads=3)
    flat_full, flat_sub = full.reshape(-1, case.d), sub.reshape(-1, case.d)
    assert np.array_equal(flat_sub[rows], flat_full[rows])
    others = np.setdiff1d(np.arange(case.B * case.Hq), rows)
    assert np.all(flat_sub[others] == 0)
    assert np.array_equal(run(case, kc, vc, nthreads=4), full)


# ---------------------------------------------------------------- special cases and invariants

def test_window_at_least_context_is_full_attention():
    case = small_case(seed=10)
    kc, vc = oracle_cache(case)
    full = run(case, kc, vc, window=0)
    for w in (100, 101, 4096):
        assert np.array_equal(run(case, kc, vc, window=w), full)
    assert not np.array_equal(run(case, kc, vc, window=99)[0], full[0])
    assert np.array_equal(run(case, kc, vc, window=99)[1:], full[1:])


def test_window_reads_only_the_last_w_positions():
    case = small_case(seed=11, window=20)
    kc, vc = oracle_cache(case)
    ref = run(case, kc, vc)
    k2, v2 = kc.copy(), vc.copy()
    off = case.offsets
    for b in range(case.B):                                   # scribble on everything outside the window
        L = int(case.seq_lens[b])
        outside = case.slot_mapping[off[b]: off[b] + max(0, L - 20)]
        k2[outside] = 0x7E
        v2[outside] = 0xFE
    assert np.array_equal(run(case, k2, v2), ref)
    inside = case.slot_mapping[off[0] + 100 - 20]
    k2[inside] ^= 0x10
    assert not np.array_equal(run(case, k2, v2)[0], ref[0])


def test_no_sink_is_plain_softmax():
    case = small_case(seed=12)
    kc, vc = oracle_cache(case)
    a = run(case, kc, vc, sinks=None)
    b = run(case, kc, vc, sinks=np.full(case.Hq, -np.inf, dtype=np.float32))
    assert np.array_equal(a, b)
    assert rel_err(a, dense_reference(case, kc, vc, sinks=None)) < 2e-5


def test_single_key_closed_form():
    case = small_case(seed=13, seq_lens=[1, 1, 1])
    kc, vc = oracle_cache(case)
    got = run(case, kc, vc, accum="f64")
    q = wl.bf16_to_f32(case.q).astype(np.float64)
    G = case.Hq // case.Hkv
    for b in range(case.B):
        slot = case.slot_mapping[b]
        for h in range(case.Hq):
            k0 = torch_decode_e4m3(kc[slot, h // G]) * case.k_scale
            v0 = torch_decode_e4m3(vc[slot, h // G]) * case.v_scale
            s0 = case.sm_scale * float(k0 @ q[b, h])
            want = v0 / (1.0 + np.exp(float(case.sinks[h]) - s0))
            assert np.allclose(got[b, h], want, rtol=1e-6, atol=1e-9)


def test_zero_query_and_equal_keys_closed_forms():
    case = small_case(seed=14)
    kc, vc = oracle_cache(case)
    G = case.Hq // case.Hkv
    off = case.offsets
    zero_q = np.zeros_like(case.q)
    got = oracle.decode_attn(kc, vc, case.P, zero_q, case.block_table, case.seq_lens, case.sinks,
                             case.sm_scale, case.k_scale, case.v_scale, accum="f64")
    for b in range(case.B):
        slots = case.slot_mapping[off[b]:off[b + 1]]
        for h in range(case.Hq):
            V = torch_decode_e4m3(vc[slots, h // G]) * case.v_scale
            want = V.sum(0) / (len(slots) + np.exp(float(case.sinks[h])))
            assert np.allclose(got[b, h], want, rtol=1e-6, atol=1e-9)
    k_same = kc.copy()
    k_same[case.slot_mapping] = kc[case.slot_mapping[0]]      # every cached key equal
    got = run(case, k_same, vc, accum="f64")
    q = wl.bf16_to_f32(case.q).astype(np.float64)
    for b in range(case.B):
        slots = case.slot_mapping[off[b]:off[b + 1]]
        for h in range(case.Hq):
            k0 = torch_decode_e4m3(k_same[slots[0], h // G]) * case.k_scale
            s0 = case.sm_scale * float(k0 @ q[b, h])
            V = torch_decode_e4m3(vc[slots, h // G]) * case.v_scale
            want = V.sum(0) / (len(slots) + np.exp(float(case.sinks[h]) - s0))
            assert np.allclose(got[b, h], want, rtol=1e-6, atol=1e-9)


def test_heads_of_a_group_with_equal_query_and_sink_agree():
    case = small_case(seed=15)
    q = case.q.copy()
    q[:, 1] = q[:, 0]
    q[:, 5] = q[:, 4]
    sinks = case.sinks.copy()
    sinks[1], sinks[5] = sinks[0], sinks[4]
    kc, vc = oracle_cache(case)
    out = oracle.decode_attn(kc, vc, case.P, q, case.block_table, case.seq_lens, sinks, case.sm_scale,
                             case.k_scale, case.v_scale)
    assert np.array_equal(out[:, 0], out[:, 1]) and np.array_equal(out[:, 4], out[:, 5])
    assert not np.array_equal(out[:, 0], out[:, 4])           # different KV head


def test_physical_page_permutation_invariance():
    case = small_case(seed=16)
    kc, vc = oracle_cache(case)
    ref = run(case, kc, vc)
    perm = np.random.default_rng(5).permutation(case.num_pages)
    P = case.P
    k2 = np.empty_like(kc).reshape(case.num_pages, P, case.Hkv, case.d)
    v2 = np.empty_like(vc).reshape(case.num_pages, P, case.Hkv, case.d)
    k2[perm] = kc.reshape(case.num_pages, P, case.Hkv, case.d)
    v2[perm] = vc.reshape(case.num_pages, P, case.Hkv, case.d)
    bt2 = np.where(case.block_table >= 0, perm[np.maximum(case.block_table, 0)], -1).astype(np.int32)
    got = oracle.decode_attn(k2.reshape(kc.shape), v2.reshape(vc.shape), P, case.q, bt2, case.seq_lens,
                             case.sinks, case.sm_scale, case.k_scale, case.v_scale)
    assert np.array_equal(got, ref)


def test_exact_scaling_properties():
    case = small_case(seed=17)
    kc, vc = oracle_cache(case)
    ref = run(case, kc, vc)
    assert np.array_equal(run(case, kc, vc, k_scale=case.k_scale * 2, sm_scale=case.sm_scale / 2), ref)
    assert np.array_equal(run(case, kc, vc, v_scale=case.v_scale * 2), ref * 2)
    big = run(case, kc, vc, sinks=np.full(case.Hq, 80.0, dtype=np.float32))
    assert np.max(np.abs(big)) < 1e-20 * np.max(np.abs(ref)) + 1e-25
    assert np.all(run(case, kc, vc, sinks=np.full(case.Hq, 200.0, dtype=np.float32)) == 0)


def test_zero_length_sequence_gives_zero_row():
    case = small_case(seed=18)
    kc, vc = oracle_cache(case)
    lens = case.seq_lens.copy()
    lens[1] = 0
    got = oracle.decode_attn(kc, vc, case.P, case.q, case.block_table, lens, case.sinks, case.sm_scale,
                             case.k_scale, case.v_scale)
    assert np.all(got[1] == 0) and np.array_equal(got[0], run(case, kc, vc)[0])


# ---------------------------------------------------------------- split-K partials and merge

@pytest.mark.parametrize("split_tokens,window", [(64, 0), (128, 0), (1024, 0), (64, 70), (128, 200)])
def test_partials_merge_to_unsplit(split_tokens, window):
    case = small_case(seed=19, seq_lens=[300, 129, 64], P=16, window=window)
    kc, vc = oracle_cache(case)
    span = 300 if window == 0 else window + 63
    S = -(-span // split_tokens)
    acc, ml = oracle.decode_attn_partials(kc, vc, case.P, case.q, case.block_table, case.seq_lens,
                                          case.sm_scale, case.k_scale, window, split_tokens, S)
    merged = oracle.splitk_reduce(acc, ml, case.sinks, case.v_scale)
    assert rel_err(merged, run(case, kc, vc, accum="f64")) < 5e-6
    assert rel_err(merged, dense_reference(case, kc, vc)) < 5e-6
    # chunk geometry: chunk i of sequence b is empty exactly when it holds no attended position
    for b in range(case.B):
        L = int(case.seq_lens[b])
        lo = L - window if (window > 0 and L > window) else 0
        a0 = lo - lo % 64
        for i in range(S):
            j0, j1 = max(a0 + i * split_tokens, lo), min(a0 + (i + 1) * split_tokens, L)
            empty = j0 >= j1
            assert np.all((ml[b, :, i, 1] == 0) == empty)
            assert np.all(np.isneginf(ml[b, :, i, 0]) == empty)
            if not empty:                                      # l counts at least the max itself
                assert np.all(ml[b, :, i, 1] >= 1.0) and np.all(ml[b, :, i, 1] <= j1 - j0)


def test_partials_of_one_chunk_against_dense():
    """A single chunk's (acc/l, m + log l) are the chunk's own softmax average and log-sum-exp."""
    case = small_case(seed=20, seq_lens=[128, 64, 100], sinks=False)
    kc, vc = oracle_cache(case)
    acc, ml = oracle.decode_attn_partials(kc, vc, case.P, case.q, case.block_table, case.seq_lens,
                                          case.sm_scale, case.k_scale, 0, 64, 2, accum="f64")
    first = dense_reference(case, kc, vc, sinks=None, seq_lens=np.minimum(case.seq_lens, 64), v_scale=1.0)
    assert rel_err(acc[:, :, 0] / ml[:, :, 0, 1:2], first) < 1e-6


def test_reduce_closed_forms():
    rng = np.random.default_rng(21)
    B, Hq, S, d = 2, 4, 3, 64
    acc = rng.standard_normal((B, Hq, S, d)).astype(np.float32)
    ml = np.stack([rng.standard_normal((B, Hq, S)) * 3, rng.uniform(1, 50, (B, Hq, S))], -1).astype(np.float32)
    sinks = rng.standard_normal(Hq).astype(np.float32)
    got = oracle.splitk_reduce(acc, ml, sinks, 0.37)
    m, l = ml[..., 0].astype(np.float64), ml[..., 1].astype(np.float64)
    w = np.exp(m)                                              # small magnitudes: no stabiliser needed
    want = 0.37 * (acc * w[..., None]).sum(2) / (np.exp(sinks.astype(np.float64))[None, :, None]
                                                 + (l * w).sum(2)[..., None])
    assert np.allclose(got, want, rtol=1e-6, atol=1e-9)
    # shifting a partial's reference maximum by c while scaling (acc, l) by exp(-c) changes nothing
    ml2, acc2 = ml.copy(), acc.copy()
    ml2[..., 0, 0] += np.float32(np.log(4.0))
    ml2[..., 0, 1] /= 4
    acc2[..., 0, :] /= 4
    assert np.allclose(oracle.splitk_reduce(acc2, ml2, sinks, 0.37), got, rtol=2e-6, atol=1e-9)
    # empty partials are ignored; all-empty without a sink is a zero row, never NaN
    ml3, acc3 = ml.copy(), acc.copy()
    ml3[:, :, 1] = (-np.inf, 0.0)
    acc3[:, :, 1] = 0
    keep = oracle.splitk_reduce(acc[:, :, [0, 2]], ml[:, :, [0, 2]], sinks, 0.37)
    assert np.allclose(oracle.splitk_reduce(acc3, ml3, sinks, 0.37), keep, rtol=1e-6, atol=1e-9)
    ml3[:, :, :] = (-np.inf, 0.0)
    acc3[:] = 0
    assert np.all(oracle.splitk_reduce(acc3, ml3, None, 1.0) == 0)
    assert np.all(oracle.splitk_reduce(acc3, ml3, sinks, 1.0) == 0)


# ---------------------------------------------------------------- multi-token (prefill) definition

def test_prefill_is_causal_attention_inside_the_window():
    """Dense float64 check of the multi-token definition: token i of the n newest sees positions
    up to its own and no more than the window before it."""
    case = small_case(seed=30, seq_lens=[90, 37, 16], P=16)
    kc, vc = oracle_cache(case)
    n_new = [40, 37, 3]
    q_start = np.concatenate([[0], np.cumsum(n_new)])
    rng = np.random.default_rng(30)
    q = wl.bf16_bits(rng.standard_normal((q_start[-1], case.Hq, case.d)).astype(np.float32))
    G = case.Hq // case.Hkv
    for window in (0, 25):
        got = oracle.prefill_attn(kc, vc, case.P, q, q_start, case.block_table, case.seq_lens, case.sinks,
                                  case.sm_scale, case.k_scale, case.v_scale, window, accum="f64")
        qf = wl.bf16_to_f32(q).astype(np.float64)
        want = np.zeros_like(got, dtype=np.float64)
        off = case.offsets
        for b in range(case.B):
            L = int(case.seq_lens[b])
            slots = case.slot_mapping[off[b]:off[b + 1]]
            for i in range(n_new[b]):
                p = L - n_new[b] + i
                lo = max(0, p - window + 1) if window else 0
                for h in range(case.Hq):
                    K = torch_decode_e4m3(kc[slots[lo:p + 1], h // G]) * case.k_scale
                    V = torch_decode_e4m3(vc[slots[lo:p + 1], h // G]) * case.v_scale
                    s = case.sm_scale * (K @ qf[q_start[b] + i, h])
                    mx = max(s.max(), float(case.sinks[h]))
                    w = np.exp(s - mx)
                    want[q_start[b] + i, h] = (w @ V) / (w.sum() + np.exp(float(case.sinks[h]) - mx))
        assert rel_err(got, want) < 1e-6
    # one new token per sequence is the decode call
    one = oracle.prefill_attn(kc, vc, case.P, case.q, np.arange(case.B + 1), case.block_table, case.seq_lens,
                              case.sinks, case.sm_scale, case.k_scale, case.v_scale, 0)
    assert np.array_equal(one, run(case, kc, vc))


def test_run_merge_helper_agrees_with_the_oracle_reduce():
    """tests/helpers.merge_runs_of_partials (used to compare workspaces whose rows hold several chunks)
    against oracle.splitk_reduce: one run over every chunk is the reduce itself, and reducing the runs'
    partials gives what reducing the chunks' partials gives."""
    from helpers import merge_runs_of_partials
    rng = np.random.default_rng(77)
    S, d = 23, 64
    acc = rng.standard_normal((S, d)).astype(np.float32)
    ml = np.stack([rng.standard_normal(S) * 15, rng.uniform(1, 500, S)], -1).astype(np.float32)
    ml[5] = (-np.inf, 0)
    ml[20:] = (-np.inf, 0)                                            # trailing chunks without positions
    want = oracle.splitk_reduce(acc[None, None], ml[None, None], None, 1.0)[0, 0]
    lse, avg = merge_runs_of_partials(acc, ml, [0])
    assert np.allclose(avg[0], want, rtol=1e-5, atol=1e-6)
    starts = [0, 4, 6, 13, 19]
    lse, avg = merge_runs_of_partials(acc, ml, starts)
    acc2 = np.zeros((S, d), dtype=np.float32)
    ml2 = np.full((S, 2), (-np.inf, 0), dtype=np.float32)
    acc2[starts] = avg
    ml2[starts, 0] = lse
    ml2[starts, 1] = 1.0
    again = oracle.splitk_reduce(acc2[None, None], ml2[None, None], None, 1.0)[0, 0]
    assert np.allclose(again, want, rtol=1e-5, atol=1e-6)
