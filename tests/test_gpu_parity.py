"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Bars: cache bytes bit-exact; attention outputs max-abs error <= 2e-3 of the oracle output's RMS
(fp32 oracle; the fp64 oracle is reported beside it)."""
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


def oracle_attn(case, kc, vc, **kw):
    a = dict(sinks=case.sinks, sm_scale=case.sm_scale, k_scale=case.k_scale, v_scale=case.v_scale,
             window=case.window, nthreads=8)
    a.update(kw)
    seq_lens = a.pop("seq_lens", case.seq_lens)
    q = a.pop("q", case.q)
    return oracle.decode_attn(kc, vc, case.P, q, case.block_table, seq_lens, **a)


# ------------------------------------------------------------------ append: bit-exact

@pytest.fixture(params=["tile", "token"])
def append_form(request, launch_override):
    """Both launch forms of the append kernel (64-token tiles / one wave per token and head)."""
    launch_override("append_form", pz.APPEND_FORM_TOKEN if request.param == "token" else pz.APPEND_FORM_TILE)
    return request.param


@pytest.mark.parametrize("P", [16, 32, 64])
@pytest.mark.parametrize("scales", ["amax", "pow2", "unit"])
def test_append_bytes_bit_exact(P, scales, append_form):
    case = wl.make_case("a", B=3, Hq=8, Hkv=2, d=64, P=P, seq_lens=[100, 37, 129], seed=P,
                        pow2_scales=scales == "pow2", unit_scales=scales == "unit", outlier_frac=0.05)
    cache = gpu_cache(case)
    gk, gv = to_oracle_layout(cache)
    ok, ov = oracle_cache(case)
    assert np.array_equal(gk, ok) and np.array_equal(gv, ov)      # includes untouched canary bytes


def test_append_every_bf16_value_and_negative_slots(append_form):
    Hkv, d, P = 2, 64, 16
    T = 65536 // (Hkv * d)
    bits = np.arange(65536, dtype=np.uint16).reshape(T, Hkv, d)
    rng = np.random.default_rng(0)
    slots = rng.permutation(T + 40)[:T].astype(np.int64)
    slots[::7] = -1
    num_pages = (T + 40 + P - 1) // P
    for k_scale, v_scale in ((1.0, 0.0123), (4.8 / 448, 2.0 ** -7), (3.0, 0.37)):
        cache = pz.PagedCache.allocate(num_pages, P, Hkv, d, pz.KV_FP8, DEV, fill=0xAA)
        pz.pz_kv_append_fp8(cache, dev_bits(bits), dev_bits(bits[::-1].copy()), torch.from_numpy(slots).to(DEV),
                            T, k_scale, v_scale)
        torch.cuda.synchronize()
        gk, gv = to_oracle_layout(cache)
        ok, ov = oracle.new_cache(num_pages * P, Hkv, d)
        oracle.kv_append(ok, ov, bits, bits[::-1].copy(), slots, k_scale, v_scale)
        nan_k = (ok & 0x7F) == 0x7F
        nan_v = (ov & 0x7F) == 0x7F
        assert nan_k.sum() > 100                                   # NaN inputs stay NaN (payload-free check)
        assert np.array_equal(gk[~nan_k], ok[~nan_k]) and np.all((gk[nan_k] & 0x7F) == 0x7F)
        assert np.array_equal(gv[~nan_v], ov[~nan_v]) and np.all((gv[nan_v] & 0x7F) == 0x7F)


def test_append_divides_on_inputs_where_the_reciprocal_product_gives_another_code(append_form):
    """Inputs whose quotient sits on a midpoint between two codes, so that x * (1 / scale) and x / scale
    quantise differently: the kernel must produce the division's code, as the oracle does."""
    from helpers import division_sensitive_inputs
    cases = division_sensitive_inputs()
    by_scale = {}
    for xb, sc, _, _ in cases:
        by_scale.setdefault(sc, []).append(xb)
    scales = sorted(by_scale, key=lambda s: -len(by_scale[s]))[:40]
    Hkv, d, P = 1, 64, 16
    n_checked = 0
    for sc in scales:
        xs = by_scale[sc]
        row = np.resize(np.array(xs, dtype=np.uint16), (1, Hkv, d))           # the scale's inputs, repeated
        neg = row | 0x8000                                                     # and their negatives for V
        cache = pz.PagedCache.allocate(1, P, Hkv, d, pz.KV_FP8, DEV, fill=0xAA)
        pz.pz_kv_append_fp8(cache, dev_bits(row), dev_bits(neg), torch.tensor([3], dtype=torch.int64, device=DEV),
                            1, sc, sc)
        torch.cuda.synchronize()
        gk, gv = to_oracle_layout(cache)
        want = oracle.quantize(row.ravel(), sc)
        assert np.array_equal(gk[3, 0], want) and np.array_equal(gv[3, 0], want | 0x80), sc
        n_checked += len(xs)
    assert n_checked >= 40


def test_append_bf16_cache_copies_bits(append_form):
    case = wl.make_case("b", B=2, Hq=8, Hkv=2, d=64, P=32, seq_lens=[70, 33], seed=1)
    cache = gpu_cache(case, dtype=pz.KV_BF16)
    gk, gv = to_oracle_layout(cache)
    ok, ov = oracle_cache(case, oracle.KV_BF16)
    assert np.array_equal(gk, ok) and np.array_equal(gv, ov)


def test_append_single_decode_token_per_sequence(append_form):
    """The decode-step shape: one new token per sequence lands in an already filled cache."""
    case = wl.make_case("c", B=5, Hq=8, Hkv=2, d=64, P=64, seq_lens=[65, 64, 1, 200, 128], seed=2)
    last = case.offsets[1:] - 1
    prefix = np.setdiff1d(np.arange(len(case.slot_mapping)), last)
    slots_prefix = case.slot_mapping.copy()
    slots_prefix[last] = -1
    cache = gpu_cache(case, slots=slots_prefix)
    pz.pz_kv_append_fp8(cache, dev_bits(case.k[last]), dev_bits(case.v[last]),
                        torch.from_numpy(case.slot_mapping[last]).to(DEV), len(last), case.k_scale, case.v_scale)
    torch.cuda.synchronize()
    gk, gv = to_oracle_layout(cache)
    ok, ov = oracle_cache(case)
    assert len(prefix) > 0 and np.array_equal(gk, ok) and np.array_equal(gv, ov)


# ------------------------------------------------------------------ attention: <= 2e-3 of RMS

CASES = {
    "cfg1_tiny": dict(B=2, Hq=8, Hkv=2, d=64, P=16, seq_lens=[100, 37], sm_scale=0.125, seed=0),
    "g8_p64_ragged": dict(B=4, Hq=16, Hkv=2, d=64, P=64, seq_lens=[1000, 64, 65, 777], seed=1),
    "g1": dict(B=3, Hq=2, Hkv=2, d=64, P=16, seq_lens=[5, 64, 170], seed=2),
    "g2_p32": dict(B=3, Hq=4, Hkv=2, d=64, P=32, seq_lens=[33, 300, 96], seed=3),
    "g8_hkv8": dict(B=2, Hq=64, Hkv=8, d=64, P=64, seq_lens=[640, 2500], seed=4),
    "window20": dict(B=3, Hq=8, Hkv=2, d=64, P=16, seq_lens=[100, 37, 19], window=20, seed=5),
    "window128_p64": dict(B=4, Hq=16, Hkv=2, d=64, P=64, seq_lens=[1000, 128, 129, 50], window=128, seed=6),
    "window_unaligned": dict(B=3, Hq=16, Hkv=2, d=64, P=64, seq_lens=[1000, 333, 4000], window=300, seed=7),
    "no_sinks": dict(B=2, Hq=8, Hkv=2, d=64, P=16, seq_lens=[100, 37], sinks=False, seed=8),
    "outliers": dict(B=2, Hq=16, Hkv=2, d=64, P=64, seq_lens=[900, 2100], outlier_frac=0.05, seed=9),
    "pow2_scales": dict(B=2, Hq=16, Hkv=2, d=64, P=64, seq_lens=[500, 70], pow2_scales=True, seed=10),
    "unit_scales": dict(B=2, Hq=16, Hkv=2, d=64, P=64, seq_lens=[500, 70], unit_scales=True, seed=11),
    "len_one_and_zero": dict(B=4, Hq=8, Hkv=2, d=64, P=16, seq_lens=[1, 2, 17, 1], seed=12),
    # groups above 8 run as 2, 4 or 8 virtual KV heads of a part of the group each
    "g16": dict(B=3, Hq=32, Hkv=2, d=64, P=64, seq_lens=[700, 64, 1300], seed=13),
    "g12_window": dict(B=2, Hq=36, Hkv=3, d=64, P=16, seq_lens=[300, 90], window=100, seed=14),
    "g10_hkv1": dict(B=2, Hq=10, Hkv=1, d=64, P=32, seq_lens=[257, 31], seed=15),
    "g32_four_virtual_heads": dict(B=2, Hq=64, Hkv=2, d=64, P=64, seq_lens=[900, 70], seed=16),
    "g24_window": dict(B=2, Hq=24, Hkv=1, d=64, P=16, seq_lens=[400, 130], window=150, seed=17),
    "g64_multi_query": dict(B=2, Hq=64, Hkv=1, d=64, P=64, seq_lens=[1500, 64], seed=18),
    # odd groups: the last part of a group is smaller (9 = 5 + 4, 11 = 6 + 5, 17 = 5 + 5 + 5 + 2) or empty (33 = 6 x 5 + 3 + 0)
    "g9": dict(B=3, Hq=18, Hkv=2, d=64, P=64, seq_lens=[700, 64, 1300], seed=19),
    "g11_window": dict(B=2, Hq=11, Hkv=1, d=64, P=16, seq_lens=[300, 90], window=100, seed=20),
    "g17": dict(B=2, Hq=34, Hkv=2, d=64, P=32, seq_lens=[257, 31], seed=21),
    "g33_empty_part": dict(B=2, Hq=33, Hkv=1, d=64, P=64, seq_lens=[900, 70], seed=22),
}


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("split_tokens", [0, 64, 256])
def test_attention_matches_oracle(name, split_tokens):
    case = wl.make_case(name, **CASES[name])
    cache = gpu_cache(case)
    kc, vc = oracle_cache(case)
    gk, gv = to_oracle_layout(cache)
    assert np.array_equal(gk, kc) and np.array_equal(gv, vc)
    want = oracle_attn(case, kc, vc)
    got = gpu_attn(case, cache, split_tokens=split_tokens)
    assert not np.any(np.isnan(got))
    e32, e64 = rel_err(got, want), rel_err(got, oracle_attn(case, kc, vc, accum="f64"))
    print("%s split=%d: err vs f32 oracle %.2e, vs f64 oracle %.2e" % (name, split_tokens, e32, e64))
    assert e32 <= TOL and e64 <= TOL


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_match_oracle(seed):
    """Seeded random geometry: heads, group size (also the two-virtual-head groups above 8), page size,
    batch, lengths (zero and one included), window, chunk length, sinks on or off."""
    rng = np.random.default_rng(1000 + seed)
    Hkv = int(rng.choice([1, 2, 3, 4, 8]))
    G = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 16]))
    P = int(rng.choice([16, 32, 64]))
    B = int(rng.integers(1, 6))
    lens = rng.integers(0, 3000 if Hkv * G <= 32 else 700, size=B)
    lens[rng.integers(0, B)] = int(rng.choice([0, 1, 63, 64, 65]))
    if lens.sum() == 0:
        lens[0] = 200
    window = int(rng.choice([0, 0, int(rng.integers(1, 2000))]))
    split = int(rng.choice([0, 64, 128, 192, 1024]))
    case = wl.make_case("r%d" % seed, B=B, Hq=Hkv * G, Hkv=Hkv, d=64, P=P, seq_lens=lens.tolist(), window=window,
                        sinks=bool(rng.integers(0, 2)), seed=2000 + seed)
    cache = gpu_cache(case)
    kc, vc = oracle_cache(case)
    want = oracle_attn(case, kc, vc, accum="f64")
    got = gpu_attn(case, cache, split_tokens=split)
    err = rel_err(got, want)
    print("seed %d: Hkv=%d G=%d P=%d lens=%s window=%d split=%d err=%.2e" % (seed, Hkv, G, P, lens.tolist(), window,
                                                                             split, err))
    assert not np.any(np.isnan(got)) and err <= TOL
    assert np.all(got[lens == 0] == 0)


def test_zero_length_rows_and_garbage_beyond_the_context():
    """L_b = 0 gives a zero row; NaN codes in cache slots outside [lo, L) never reach the output."""
    case = wl.make_case("z", B=4, Hq=8, Hkv=2, d=64, P=16, seq_lens=[100, 37, 64, 9], seed=13)
    cache = gpu_cache(case, fill=0x7F)                             # unwritten slots decode to NaN
    kc, vc = oracle_cache(case)
    lens = np.array([100, 0, 50, 9], dtype=np.int32)               # shorter than what was appended
    for window, split in ((0, 0), (0, 64), (24, 0), (24, 64)):
        want = oracle_attn(case, kc, vc, seq_lens=lens, window=window)
        got = gpu_attn(case, cache, seq_lens=lens, window=window, split_tokens=split)
        assert np.all(got[1] == 0) and not np.any(np.isnan(got))
        assert rel_err(got, want) <= TOL
    # positions before the window start hold NaN codes too
    k2 = case.k.copy()
    off = case.offsets
    k2[off[0]:off[0] + 70] = 0x7FC0                                 # bf16 NaN -> E4M3 NaN
    case2 = wl.Case(**{**case.__dict__, "k": k2, "v": k2})
    cache2 = gpu_cache(case2, fill=0x7F)
    kc2, vc2 = oracle_cache(case2)
    want = oracle_attn(case2, kc2, vc2, window=24)
    got = gpu_attn(case2, cache2, window=24)
    assert not np.any(np.isnan(want)) and not np.any(np.isnan(got)) and rel_err(got, want) <= TOL


def test_special_cases_on_gpu():
    case = wl.make_case("s", B=3, Hq=16, Hkv=2, d=64, P=64, seq_lens=[300, 64, 1], seed=14)
    cache = gpu_cache(case)
    full = gpu_attn(case, cache, window=0)
    assert np.array_equal(gpu_attn(case, cache, window=300), full)          # window >= L is full attention
    assert np.array_equal(gpu_attn(case, cache, window=100000), full)
    a = gpu_attn(case, cache, sinks=None)
    b = gpu_attn(case, cache, sinks=np.full(case.Hq, -np.inf, dtype=np.float32))
    assert np.array_equal(a, b)                                             # sink = -inf is plain softmax
    kc, vc = oracle_cache(case)
    assert rel_err(a, oracle_attn(case, kc, vc, sinks=None)) <= TOL
    assert np.array_equal(gpu_attn(case, cache, v_scale=case.v_scale * 2), full * 2)
    big = gpu_attn(case, cache, sinks=np.full(case.Hq, 300.0, dtype=np.float32))
    assert np.all(big == 0)
    assert np.array_equal(gpu_attn(case, cache), full)                      # deterministic


def test_bf16_output_is_one_rounding_of_the_fp32_result():
    case = wl.make_case("o", B=2, Hq=16, Hkv=2, d=64, P=64, seq_lens=[300, 70], seed=15)
    cache = gpu_cache(case)
    f32 = gpu_attn(case, cache)
    for split in (0, 128):
        b16 = gpu_attn(case, cache, split_tokens=split, out_dtype=pz.OUT_BF16)
        want = torch.from_numpy(gpu_attn(case, cache, split_tokens=split)).to(torch.bfloat16).float().numpy()
        assert np.array_equal(b16, want)
    assert rel_err(gpu_attn(case, cache, out_dtype=pz.OUT_BF16), f32) < 8e-3


def test_bf16_kv_cache_variant():
    case = wl.make_case("k", B=3, Hq=16, Hkv=2, d=64, P=64, seq_lens=[700, 64, 130], seed=16)
    cache = gpu_cache(case, dtype=pz.KV_BF16)
    kb, vb = oracle_cache(case, oracle.KV_BF16)
    want = oracle_attn(case, kb, vb, k_scale=1.0, v_scale=1.0)
    for split, window in ((0, 0), (128, 0), (0, 100), (64, 100)):
        want = oracle_attn(case, kb, vb, k_scale=1.0, v_scale=1.0, window=window)
        got = gpu_attn(case, cache, k_scale=1.0, v_scale=1.0, split_tokens=split, window=window)
        assert rel_err(got, want) <= TOL
    case16 = wl.make_case("k16", B=2, Hq=8, Hkv=2, d=64, P=16, seq_lens=[100, 37], seed=17)
    cache16 = gpu_cache(case16, dtype=pz.KV_BF16)
    kb, vb = oracle_cache(case16, oracle.KV_BF16)
    got = gpu_attn(case16, cache16, k_scale=1.0, v_scale=1.0)
    assert rel_err(got, oracle_attn(case16, kb, vb, k_scale=1.0, v_scale=1.0)) <= TOL


# ------------------------------------------------------------------ split-K pieces

def test_partials_match_the_chunked_oracle():
    """Workspace contents against the oracle's chunked definition: what is unique about a partial
    is acc/l (the softmax average of its positions) and m + log l (their log-sum-exp); a row holds the
    partial of a run of chunks (the following rows of the run are empty), and chunks without an
    attended position are left unwritten."""
    case = wl.make_case("p", B=3, Hq=16, Hkv=2, d=64, P=64, seq_lens=[1000, 130, 64], window=0, seed=18)
    cache = gpu_cache(case)
    kc, vc = oracle_cache(case)
    for window, split in ((0, 256), (0, 64), (200, 128)):
        S = pz.pz_decode_attn_n_splits(1000, window, split)
        _, acc, ml = gpu_attn(case, cache, window=window, split_tokens=split, return_ws=True)
        oacc, oml = oracle.decode_attn_partials(kc, vc, case.P, case.q, case.block_table, case.seq_lens,
                                                case.sm_scale, case.k_scale, window, split, S, accum="f64")
        empty = np.isneginf(oml[..., 0])                            # chunks beyond a context: never written
        assert np.all(np.isnan(acc[empty]))
        assert check_workspace_rows(acc, ml, oacc, oml, TOL) >= case.B * case.Hq


def test_one_chunk_per_workgroup_writes_one_partial_per_chunk(launch_override):
    """With several waves per workgroup a workgroup holds one chunk, so every chunk with a position has
    a partial of its own: the per-chunk form of the workspace, compared row by row."""
    launch_override("attn_waves", 2)
    case = wl.make_case("pc", B=2, Hq=16, Hkv=2, d=64, P=64, seq_lens=[1000, 300], seed=28)
    cache = gpu_cache(case)
    kc, vc = oracle_cache(case)
    S = pz.pz_decode_attn_n_splits(1000, 0, 128)
    _, acc, ml = gpu_attn(case, cache, split_tokens=128, return_ws=True)
    oacc, oml = oracle.decode_attn_partials(kc, vc, case.P, case.q, case.block_table, case.seq_lens,
                                            case.sm_scale, case.k_scale, 0, 128, S, accum="f64")
    live = oml[..., 0] > -np.inf
    assert np.array_equal(np.isfinite(ml[..., 0]), live)
    assert check_workspace_rows(acc, ml, oacc, oml, TOL) == int(live.sum())


@pytest.mark.parametrize("S", [7, 64, 65, 128, 130, 256, 300, 513, 1100])
def test_reduce_kernel_alone_against_oracle_reduce(S):
    """The merge on synthetic partials; 64 chunks per wave, so the counts cover one to eight waves per row,
    full and ragged last batches, and waves that see only empty partials."""
    rng = np.random.default_rng(19 + S)
    B, Hq, d = 4, 16, 64
    acc = rng.standard_normal((B, Hq, S, d)).astype(np.float32)
    ml = np.stack([rng.standard_normal((B, Hq, S)) * 20, rng.uniform(1, 900, (B, Hq, S))], -1).astype(np.float32)
    ml[0, :, 3] = (-np.inf, 0)
    acc[0, :, 3] = 0
    ml[1] = (-np.inf, 0)                                            # a row with only empty partials
    acc[1] = 0
    ml[2, :, :max(1, S - 70)] = (-np.inf, 0)                        # only the last batches hold anything
    acc[2, :, :max(1, S - 70)] = 0
    ml[3, :, S // 2:] = (-np.inf, 0)                                # only the first ones do
    acc[3, :, S // 2:] = 0
    sinks = rng.standard_normal(Hq).astype(np.float32)
    ws = torch.from_numpy(np.concatenate([acc.ravel(), ml.ravel()])).to(DEV)
    for sk in (sinks, None):
        out = torch.full((B, Hq, d), float("nan"), device=DEV)
        skd = None if sk is None else torch.from_numpy(sk).to(DEV)
        pz.pz_decode_attn_splitk_reduce(ws, ws.numel() * 4, B, Hq, d, S, None, 0, 0, skd, 0.37, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        want = oracle.splitk_reduce(acc, ml, sk, 0.37)
        assert np.all(got[1] == 0) and not np.any(np.isnan(got))
        assert rel_err(got, want) < 1e-5


def test_split_count_invariance():
    case = wl.make_case("i", B=2, Hq=16, Hkv=2, d=64, P=64, seq_lens=[4000, 1500], seed=20)
    cache = gpu_cache(case)
    kc, vc = oracle_cache(case)
    want = oracle_attn(case, kc, vc, accum="f64")
    outs = [gpu_attn(case, cache, split_tokens=s) for s in (0, 64, 576, 1024, 4096)]
    for o in outs:
        assert rel_err(o, want) <= TOL
        assert rel_err(o, outs[0]) < 1e-4
    more = gpu_attn(case, cache, split_tokens=1024, n_splits=9)     # surplus chunks are ignored
    assert rel_err(more, outs[3]) < 1e-6


# ------------------------------------------------------------------ launch shapes

@pytest.mark.parametrize("B,max_len,split", [(150, 400, 64), (70, 3000, 256), (64, 900, 128), (65, 130, 64),
                                             (300, 64, 64), (5, 20000, 1024)])
def test_balanced_partition_over_many_ragged_sequences(B, max_len, split, launch_override):
    """Full-attention split-K deals the chunks of the whole batch out evenly: batches beyond one
    64-lane strip of lengths, shares that span several sequences, sequences without a token, and
    (forced by one wave per workgroup) totals far below the number of workgroups."""
    launch_override("attn_waves", 1)
    rng = np.random.default_rng(B + split)
    lens = rng.integers(0, max_len + 1, size=B)
    lens[rng.integers(0, B, size=max(1, B // 10))] = 0
    lens[-1] = max_len
    case = wl.make_case("bal", B=B, Hq=8, Hkv=2, d=64, P=64, seq_lens=lens.tolist(), seed=B)
    cache = gpu_cache(case)
    kc, vc = oracle_cache(case)
    want = oracle_attn(case, kc, vc, accum="f64")
    got, acc, ml = gpu_attn(case, cache, split_tokens=split, return_ws=True)
    assert not np.any(np.isnan(got)) and rel_err(got, want) <= TOL
    assert np.all(got[lens == 0] == 0)
    # every chunk that holds a position was written (as a partial or as an empty row of a run), no other
    # row was, and every partial is the oracle's merge of its run of chunks
    for b in range(B):
        n_b = -(-int(lens[b]) // split)
        assert not np.any(np.isnan(ml[b, :, :n_b])) and np.all(np.isnan(ml[b, :, n_b:]))
    oacc, oml = oracle.decode_attn_partials(kc, vc, case.P, case.q, case.block_table, case.seq_lens, case.sm_scale,
                                            case.k_scale, 0, split, ml.shape[2], accum="f64", nthreads=8)
    n_partials = check_workspace_rows(acc, ml, oacc, oml, TOL)
    assert n_partials >= int((lens > 0).sum()) * case.Hq


@pytest.mark.parametrize("B,Hq,Hkv", [(8, 8, 2), (6, 6, 3)])
def test_balanced_partition_with_long_shares(B, Hq, Hkv):
    """So many chunks that a share of one wave per SIMD holds 20 and more of them and crosses several
    sequences, also with a head count that does not divide the SIMD count."""
    rng = np.random.default_rng(B * Hkv)
    lens = rng.integers(50000, 131073, size=B)
    lens[0] = 131072
    split = 64
    assert sum(-(-int(L) // split) for L in lens) * Hkv > 18 * 1024
    case = wl.make_case("long_shares", B=B, Hq=Hq, Hkv=Hkv, d=64, P=64, seq_lens=lens.tolist(), seed=B)
    cache = gpu_cache(case)
    kc, vc = oracle_cache(case)
    want = oracle_attn(case, kc, vc, accum="f64")
    got, acc, ml = gpu_attn(case, cache, split_tokens=split, return_ws=True)
    assert not np.any(np.isnan(got)) and rel_err(got, want) <= TOL
    for b in range(B):
        n_b = -(-int(lens[b]) // split)
        assert not np.any(np.isnan(ml[b, :, :n_b])) and np.all(np.isnan(ml[b, :, n_b:]))


@pytest.mark.parametrize("B,expected_runs", [(130, 1), (70, 3), (32, 6)])
def test_window_split_groups_of_chunks(B, expected_runs):
    """Window layers with enough (sequence, KV head) pairs that a one-wave workgroup walks several chunks:
    the whole window (130 sequences x 8 heads fill the SIMDs) or pairs of chunks; with few pairs a chunk
    is dealt to several waves and every chunk has its partial.  A window of 300 positions in 64-token
    chunks is 4 whole chunks and up to two short ones."""
    rng = np.random.default_rng(B)
    lens = rng.integers(1, 900, size=B)
    lens[:3] = (899, 300, 64)
    case = wl.make_case("wg", B=B, Hq=8, Hkv=8, d=64, P=64, seq_lens=lens.tolist(), window=300, seed=B)
    cache = gpu_cache(case)
    kc, vc = oracle_cache(case)
    want = oracle_attn(case, kc, vc, accum="f64")
    got, acc, ml = gpu_attn(case, cache, split_tokens=64, return_ws=True)
    assert not np.any(np.isnan(got)) and rel_err(got, want) <= TOL
    oacc, oml = oracle.decode_attn_partials(kc, vc, case.P, case.q, case.block_table, case.seq_lens, case.sm_scale,
                                            case.k_scale, 300, 64, ml.shape[2], accum="f64", nthreads=8)
    check_workspace_rows(acc, ml, oacc, oml, TOL)
    # the longest sequence: its 6 chunks form the expected number of runs
    assert int(np.isfinite(ml[0, 0, :, 0]).sum()) == expected_runs


def test_balanced_partition_degenerate_batches(launch_override):
    """No chunk at all (every sequence empty), a single sequence, and one chunk for the whole batch."""
    launch_override("attn_waves", 1)
    for lens, split in (([0, 0, 0], 64), ([777], 64), ([5], 1024), ([0, 3, 0, 0], 128), ([64] * 70, 64)):
        case = wl.make_case("deg", B=len(lens), Hq=8, Hkv=2, d=64, P=16, seq_lens=lens, seed=len(lens))
        cache = gpu_cache(case)
        kc, vc = oracle_cache(case)
        want = oracle_attn(case, kc, vc, accum="f64")
        got = gpu_attn(case, cache, split_tokens=split, n_splits=max(1, -(-max(lens) // split)))
        assert not np.any(np.isnan(got))
        if max(lens) == 0:
            assert np.all(got == 0)
        else:
            assert rel_err(got, want) <= TOL


@pytest.mark.parametrize("lens,split,window", [
    ("many_short", 64, 0),                   # 1024 sequences of 0..200 tokens: 16 strips of lengths in the partition
    ([131072], 64, 0),                       # one sequence, 2048 chunks
    ([100000, 5], 65536, 0),                 # chunks longer than most contexts
    ([131072, 70000], 1024, 8192),           # window layer at the longest context
    ([500, 64, 63, 1], 64, 1),               # a window of one token: the newest token alone
    ([500, 64, 65, 1], 64, 63), ([500, 64, 65, 1], 64, 64), ([500, 64, 65, 1], 0, 65),
])
def test_extreme_shapes(lens, split, window):
    if lens == "many_short":
        rng = np.random.default_rng(1024)
        lens = rng.integers(0, 201, size=1024).tolist()
    case = wl.make_case("x", B=len(lens), Hq=8, Hkv=2, d=64, P=64, seq_lens=lens, window=window, seed=len(lens) + window)
    cache = gpu_cache(case)
    kc, vc = oracle_cache(case)
    want = oracle_attn(case, kc, vc, accum="f64")
    got = gpu_attn(case, cache, split_tokens=split)
    assert not np.any(np.isnan(got)) and rel_err(got, want) <= TOL
    if window == 1:                           # softmax over one logit and the sink
        assert np.all(got[np.asarray(lens) == 0] == 0)


@pytest.mark.parametrize("P", [16, 32, 64])
@pytest.mark.parametrize("window", [1, 20, 64, 128, 129])
@pytest.mark.parametrize("kv_dtype", [pz.KV_FP8, pz.KV_BF16])
def test_short_windows_single_pass(P, window, kv_dtype):
    """Single-pass calls over one to three steps: every alignment of a short window against the 64-position
    steps, contexts shorter than the window, empty sequences, both cache types and both output types."""
    lens = [0, 1, 63, 64, 65, 127, 128, 129, 191, 192, 193, 255, 256, 257, 1000, 1001, 4033]
    case = wl.make_case("sw", B=len(lens), Hq=16, Hkv=2, d=64, P=P, seq_lens=lens, window=window, seed=window + P)
    ks, vs = (case.k_scale, case.v_scale) if kv_dtype == pz.KV_FP8 else (1.0, 1.0)
    cache = gpu_cache(case, dtype=kv_dtype, k_scale=ks, v_scale=vs)
    kc, vc = oracle_cache(case, oracle.KV_FP8 if kv_dtype == pz.KV_FP8 else oracle.KV_BF16)
    want = oracle_attn(case, kc, vc, k_scale=ks, v_scale=vs, accum="f64")
    got = gpu_attn(case, cache, k_scale=ks, v_scale=vs)
    assert not np.any(np.isnan(got)) and rel_err(got, want) <= TOL and np.all(got[0] == 0)
    b16 = gpu_attn(case, cache, k_scale=ks, v_scale=vs, out_dtype=pz.OUT_BF16)
    assert np.array_equal(b16, torch.from_numpy(got).to(torch.bfloat16).float().numpy())


def test_short_contexts_without_a_window():
    """Full attention, single pass, over contexts of at most 192 positions (a block table of three steps)."""
    case = wl.make_case("sc", B=5, Hq=24, Hkv=2, d=64, P=16, seq_lens=[192, 1, 100, 0, 129], seed=31)
    cache = gpu_cache(case)
    kc, vc = oracle_cache(case)
    assert case.max_pages * case.P <= 192
    got = gpu_attn(case, cache)
    assert rel_err(got, oracle_attn(case, kc, vc, accum="f64")) <= TOL


@pytest.mark.parametrize("waves,cpg,balanced", [(1, 1, 0), (1, 2, 0), (1, 3, 0), (1, 8, 0), (1, 1, 1), (2, 1, 1),
                                                (4, 1, 1), (8, 1, 1)])
def test_every_launch_shape_gives_the_same_answer(waves, cpg, balanced, launch_override):
    """Waves per workgroup, chunks per workgroup and the balanced partition of full-attention split-K
    are launch heuristics; force each shape."""
    launch_override("attn_waves", waves)
    launch_override("attn_chunks_per_group", cpg)
    launch_override("attn_balanced", balanced)
    case = wl.make_case("l", B=3, Hq=16, Hkv=2, d=64, P=64, seq_lens=[2000, 130, 700], seed=21)
    cache = gpu_cache(case)
    kc, vc = oracle_cache(case)
    for window in (0, 300):
        want = oracle_attn(case, kc, vc, window=window, accum="f64")
        for split in (0, 128, 320):
            got = gpu_attn(case, cache, window=window, split_tokens=split)
            assert not np.any(np.isnan(got)) and rel_err(got, want) <= TOL, (window, split)
        # chunks beyond a context are not written (the NaN canary of the workspace stays) and the
        # merge ignores them; the chunks that hold attended positions are all written
        got, acc, ml = gpu_attn(case, cache, window=window, split_tokens=128, n_splits=19, return_ws=True)
        assert not np.any(np.isnan(got)) and rel_err(got, want) <= TOL
        for b in range(case.B):
            lo = max(0, int(case.seq_lens[b]) - window) if window else 0
            n_b = -(-(int(case.seq_lens[b]) - (lo - lo % 64)) // 128)
            assert np.all(np.isnan(ml[b, :, n_b:])) and np.all(np.isnan(acc[b, :, n_b:]))
            assert not np.any(np.isnan(ml[b, :, :n_b]))
        # and every row is the oracle's partial of its run of chunks (one chunk, or the chunks a
        # one-wave workgroup walks)
        oacc, oml = oracle.decode_attn_partials(kc, vc, case.P, case.q, case.block_table, case.seq_lens,
                                                case.sm_scale, case.k_scale, window, 128, 19, accum="f64")
        n_partials = check_workspace_rows(acc, ml, oacc, oml, TOL)
        if waves > 1 or (cpg == 1 and not balanced):
            assert n_partials == int((oml[..., 0] > -np.inf).sum())      # one chunk per workgroup
