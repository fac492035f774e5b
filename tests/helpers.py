"""Test-side helpers: an independent dense float64 reference and oracle cache construction.

The dense reference below is written from the textbook definition of softmax attention with
numpy/torch library routines (float8 decoding by torch.float8_e4m3fn, softmax by scipy); it
shares no code with oracle/pz_oracle.c and is what pins it.
"""
import numpy as np
import torch
from scipy.special import logsumexp

import oracle
from workloads import Case, bf16_to_f32


def torch_decode_e4m3(codes: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(np.ascontiguousarray(codes, dtype=np.uint8))
    return t.view(torch.float8_e4m3fn).to(torch.float64).numpy()


def oracle_cache(case: Case, kv_dtype=oracle.KV_FP8, upto=None):
    """Oracle-layout caches filled by the oracle's own append from the case's bf16 K/V."""
    kc, vc = oracle.new_cache(case.num_pages * case.P, case.Hkv, case.d, kv_dtype)
    n = len(case.slot_mapping) if upto is None else upto
    oracle.kv_append(kc, vc, case.k[:n], case.v[:n], case.slot_mapping[:n], case.k_scale, case.v_scale)
    return kc, vc


def dense_reference(case: Case, kc, vc, window=None, sinks="case", sm_scale=None, k_scale=None,
                    v_scale=None, seq_lens=None):
    """float64 softmax attention over the dequantised cache, dense, one (b, h) at a time."""
    window = case.window if window is None else window
    sinks = case.sinks if isinstance(sinks, str) else sinks
    sm_scale = case.sm_scale if sm_scale is None else sm_scale
    k_scale = case.k_scale if k_scale is None else k_scale
    v_scale = case.v_scale if v_scale is None else v_scale
    seq_lens = case.seq_lens if seq_lens is None else seq_lens
    G = case.Hq // case.Hkv
    dec = torch_decode_e4m3 if kc.dtype == np.uint8 else (lambda b: bf16_to_f32(b).astype(np.float64))
    q = bf16_to_f32(case.q).astype(np.float64)
    out = np.zeros((case.B, case.Hq, case.d))
    for b in range(case.B):
        L = int(seq_lens[b])
        if L == 0:
            continue
        lo = L - window if (window > 0 and L > window) else 0
        j = np.arange(lo, L)
        slots = case.block_table[b, j // case.P].astype(np.int64) * case.P + j % case.P
        for h in range(case.Hq):
            g = h // G
            K = dec(kc[slots, g, :]) * k_scale            # [n][d]
            V = dec(vc[slots, g, :]) * v_scale
            s = sm_scale * (K @ q[b, h])
            logits = s if sinks is None else np.concatenate([s, [float(sinks[h])]])
            p = np.exp(logits - logsumexp(logits))
            out[b, h] = p[:len(s)] @ V
    return out


def rel_err(got, want):
    """max-abs error relative to the RMS of the reference output (the parity metric)."""
    want = np.asarray(want, dtype=np.float64)
    rms = np.sqrt(np.mean(want ** 2))
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - want)) / (rms if rms > 0 else 1.0))


def paper_values():
    """The values the paper prints (tests/golden/paper_values.txt) as a dict of floats."""
    import os
    out = {}
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_values.txt")) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if line:
                key, val = (x.strip() for x in line.split("=", 1))
                out[key] = float(val)
    return out


def division_sensitive_inputs():
    """(bf16 bits of x, scale, fl(x / scale), fl(x * fl(1 / scale))) where the two quotients quantise to
    different E4M3 codes: for a bf16 x in [1, 4) and the midpoint between two adjacent codes, scales
    within a few ulps of x / midpoint put the quotient on or beside the midpoint, where one ulp decides
    the code.  Quotients by numpy's IEEE fp32 arithmetic, codes by PyTorch's float8 conversion."""
    import torch
    from workloads import bf16_bits, bf16_to_f32

    def code_value(c):
        e, m = (c >> 3) & 15, c & 7
        return m * 2.0 ** -9 if e == 0 else (8 + m) * 2.0 ** (e - 10)

    x = bf16_to_f32(np.arange(0x3F80, 0x4080, dtype=np.uint16))
    found = []
    for code in range(0x30, 0x60):                                  # midpoints above the codes of 0.25 .. 28
        mid = np.float32((code_value(code) + code_value(code + 1)) / 2)
        s0 = (x / mid).astype(np.float32)
        for ds in range(-3, 4):
            sc = (s0.view(np.int32) + np.int32(ds)).view(np.float32)
            r1 = x / sc
            r2 = x * (np.float32(1.0) / sc)
            idx = np.nonzero(r1 != r2)[0]
            c1 = torch.from_numpy(r1[idx]).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
            c2 = torch.from_numpy(r2[idx]).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
            for i in idx[c1 != c2]:
                found.append((int(bf16_bits(x[i:i + 1])[0]), float(sc[i]), float(r1[i]), float(r2[i])))
    return found


def merge_runs_of_partials(oacc, oml, starts):
    """Per-chunk partials of one (sequence, head) row -> one partial per run of consecutive chunks.

    oacc [S][d], oml [S][2] = (m, l) per chunk; `starts` = sorted chunk indices at which a run begins,
    run i covering [starts[i], starts[i + 1]) and the last one every chunk up to the last non-empty one.
    Returns (lse [R], avg [R][d]): the log-sum-exp of a run's logits and its softmax average of V,
    the two quantities of a partial that do not depend on the reference maximum."""
    oacc = np.asarray(oacc, dtype=np.float64)
    m = np.asarray(oml[:, 0], dtype=np.float64)
    l = np.asarray(oml[:, 1], dtype=np.float64)
    live = np.nonzero(m > -np.inf)[0]
    end_all = int(live[-1]) + 1 if len(live) else 0
    lse, avg = [], []
    for i, a in enumerate(starts):
        b = starts[i + 1] if i + 1 < len(starts) else end_all
        mm, ll, aa = m[a:b], l[a:b], oacc[a:b]
        M = mm.max()
        w = np.where(mm > -np.inf, np.exp(mm - M), 0.0)
        den = float((ll * w).sum())
        lse.append(M + np.log(den))
        avg.append((aa * w[:, None]).sum(axis=0) / den)
    return np.array(lse), np.array(avg)


def check_workspace_rows(acc, ml, oacc, oml, tol, lse_tol=1e-4):
    """The split-K workspace of the GPU path ([B][Hq][S][d] and [B][Hq][S][2]) against the oracle's
    per-chunk partials.  A row is unwritten (chunk without an attended position), empty (m = -inf,
    l = 0: its chunk was merged into an earlier row) or holds the partial of the run of chunks from
    itself to the next row that is not empty.  Returns the number of rows that hold a partial.

    Two quantities of a partial do not depend on its reference maximum: acc / l (bar: `tol`, the
    output tolerance) and the log-sum-exp m + ln l.  The bound on the latter, 1e-4 in natural-log
    units, follows from the kernel's arithmetic against an exact evaluation (the oracle side is
    accumulated in fp64 and stored as fp32: 2e-6):
      * each weight p_j enters l as two truncated bf16 terms, 16 significant bits: a one-sided
        relative deficit below 2^-15 per term, so ln l is low by at most 3.1e-5;
      * a logit is an fp32 sum of 64 exact products, scaled by the fp32 constant
        sm_scale * k_scale * log2(e) (two roundings) inside one fused multiply-add: at most
        (64 + 3) * 2^-24 of sum_c |q_c k_c| * sm_scale * k_scale, which is 4e-6 per unit of that sum;
        the test cases keep the sum below 10 for the positions that carry weight: 4e-5;
      * the hardware exp2 (1 ulp), the rescaling of l by exp2(m_old - m_new) once per 64 positions
        (a rounding each, at most 128 of them in these cases) and m * ln 2 in fp32: 1.5e-5 together.
    The three add up to 8.6e-5 in the worst case, all signs aligned.  With 128-channel heads a logit is a
    sum of 128 products ((128 + 3) * 2^-24 = 7.8e-6 per unit of a sum that stays below 10: 7.8e-5), 1.24e-4 in
    all: those cases pass lse_tol = 1.5e-4."""
    B, Hq, S, _ = acc.shape
    n_partials = 0
    worst_avg, worst_lse = 0.0, 0.0
    for b in range(B):
        for h in range(Hq):
            gm, gl = ml[b, h, :, 0], ml[b, h, :, 1]
            o_live = oml[b, h, :, 0] > -np.inf
            assert np.all(np.isnan(gm[~o_live])), "a chunk without positions was written"
            assert not np.any(np.isnan(gm[o_live])), "a chunk with positions was not written"
            if not o_live.any():
                continue
            starts = [int(i) for i in np.nonzero(np.isfinite(gm))[0]]
            assert starts and starts[0] == int(np.nonzero(o_live)[0][0]), "the first chunk must hold a partial"
            empty_rows = o_live & ~np.isfinite(gm)
            assert np.all(np.isneginf(gm[empty_rows])) and np.all(gl[empty_rows] == 0)
            lse_o, avg_o = merge_runs_of_partials(oacc[b, h], oml[b, h], starts)
            lse_g = gm[starts].astype(np.float64) + np.log(gl[starts].astype(np.float64))
            avg_g = acc[b, h][starts].astype(np.float64) / gl[starts].astype(np.float64)[:, None]
            worst_lse = max(worst_lse, float(np.max(np.abs(lse_g - lse_o))))
            rms = float(np.sqrt(np.mean(avg_o ** 2)))
            worst_avg = max(worst_avg, float(np.max(np.abs(avg_g - avg_o))) / (rms if rms > 0 else 1.0))
            n_partials += len(starts)
    assert worst_lse < lse_tol, worst_lse
    assert worst_avg <= tol, worst_avg
    return n_partials
