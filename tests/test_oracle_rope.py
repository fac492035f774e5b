"""Pins of the oracle's YaRN rotary tables and of its fused rotary + append (CPU only).

What the paper fixes: the parent's YaRN encoding is kept and its scaling factor goes from 32 to
56 (Section 2).  The rest is the published YaRN rule; the checks below are its defining
properties (written with numpy float64, independent of the oracle's code): factor 1 is plain
rotary embedding; pairs that turn at least beta_fast times over the original context keep their
frequency; pairs that turn at most beta_slow times are interpolated by the factor; in between the
blend is linear in the pair index; cos/sin carry the temperature 0.1 ln(factor) + 1; a rotation
preserves norms and makes q.k a function of the position difference only.

parity unpinned: the paper prints only the factor.  The temperature term, theta, beta_fast, beta_slow
and the original context are the published YaRN rule with the parent model's public configuration;
nothing in the paper confirms them, so the checks of those below restate the reading, they do not pin
it.  This file imports nothing of the HIP library."""
import numpy as np
import torch

import oracle
from helpers import paper_values, torch_decode_e4m3
from workloads import bf16_bits, bf16_to_f32

D, THETA, L0 = 64, 150000.0, 4096


def test_defaults_are_the_papers_yarn_factor_and_contexts():
    pv = paper_values()
    assert pv["yarn_factor"] == 56 and pv["yarn_factor_parent"] == 32
    # 32 is the nominal extension ratio of the parent: original context x 32 = extended context
    assert pv["yarn_original_context"] * pv["yarn_factor_parent"] == pv["yarn_extended_context"]
    assert pv["yarn_original_context"] == L0
    c_def, s_def = oracle.yarn_table(D, 3)
    c_56, s_56 = oracle.yarn_table(D, 3, theta=THETA, factor=pv["yarn_factor"], original_context=L0)
    assert np.array_equal(c_def, c_56) and np.array_equal(s_def, s_56)


def angles(cos, sin, t):
    return np.arctan2(sin.astype(np.float64) / t, cos.astype(np.float64) / t)


def test_factor_one_is_plain_rotary_embedding():
    cos, sin = oracle.yarn_table(D, 300, theta=THETA, factor=1.0)
    p = np.arange(300)[:, None]
    f = THETA ** (-2.0 * np.arange(D // 2) / D)[None, :]
    assert np.allclose(cos, np.cos(p * f), atol=2e-7) and np.allclose(sin, np.sin(p * f), atol=2e-7)


def test_yarn_blend_temperature_and_factor():
    for factor in (32.0, 56.0):
        cos, sin = oracle.yarn_table(D, 2, theta=THETA, factor=factor, original_context=L0)
        t = 0.1 * np.log(factor) + 1.0
        assert np.allclose(cos[0], t, rtol=1e-7) and np.all(sin[0] == 0)
        assert np.allclose(cos.astype(np.float64) ** 2 + sin.astype(np.float64) ** 2, t * t, rtol=1e-6)
        inv = angles(cos, sin, t)[1]                                  # angle at position 1 = frequency
        f = THETA ** (-2.0 * np.arange(D // 2) / D)
        rot = L0 * f / (2 * np.pi)                                    # turns over the original context
        fast, slow = rot >= 32.0, rot <= 1.0
        assert fast.sum() > 5 and slow.sum() > 5 and (~fast & ~slow).sum() > 3
        assert np.allclose(inv[fast], f[fast], rtol=1e-5)            # extrapolated: unchanged
        assert np.allclose(inv[slow], f[slow] / factor, rtol=1e-5)   # interpolated by the factor
        mid = np.where(~fast & ~slow)[0]
        w = (f[mid] - inv[mid]) / (f[mid] - f[mid] / factor)         # weight of the interpolated frequency
        assert np.all(np.diff(w) > 0) and np.all((w > 0) & (w < 1))
        assert np.allclose(np.diff(w), np.diff(w)[0], rtol=1e-3)     # linear in the pair index
        assert np.all(np.diff(inv) < 0)
    c56, _ = oracle.yarn_table(D, 2, factor=56.0)
    c32, _ = oracle.yarn_table(D, 2, factor=32.0)
    assert not np.allclose(c56, c32)


def rotate_f64(x, cos, sin):
    h = x.shape[-1] // 2
    x1, x2 = x[..., :h], x[..., h:]
    return np.concatenate([x1 * cos - x2 * sin, x2 * cos + x1 * sin], -1)


def make_inputs(T=9, Hq=8, Hkv=2, seed=0):
    rng = np.random.default_rng(seed)
    q = bf16_bits(rng.standard_normal((T, Hq, D)).astype(np.float32))
    k = bf16_bits(rng.standard_normal((T, Hkv, D)).astype(np.float32))
    v = bf16_bits(rng.standard_normal((T, Hkv, D)).astype(np.float32))
    pos = rng.integers(0, 3000, T).astype(np.int32)
    slots = rng.permutation(T + 7)[:T].astype(np.int64)
    return q, k, v, pos, slots


def test_rope_append_matches_float64_rotation_and_quantisation():
    q, k, v, pos, slots = make_inputs()
    cos, sin = oracle.yarn_table(D, 3000)
    k_scale, v_scale = 6.5 / 448, 4.5 / 448
    kc, vc = oracle.new_cache(16, 2, D)
    q_out = oracle.rope_kv_append(kc, vc, q, k, v, pos, cos, sin, slots, k_scale, v_scale)
    c, s = cos[pos][:, None, :].astype(np.float64), sin[pos][:, None, :].astype(np.float64)
    want_q = rotate_f64(bf16_to_f32(q).astype(np.float64), c, s)
    got_q = bf16_to_f32(q_out).astype(np.float64)
    assert np.max(np.abs(got_q - want_q)) <= 2.0 ** -8 * np.max(np.abs(want_q))     # one bf16 rounding
    tq = torch.from_numpy(want_q.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.mean(tq == q_out) > 0.999
    want_k = rotate_f64(bf16_to_f32(k).astype(np.float64), c, s) / k_scale
    tk = torch.from_numpy(want_k.astype(np.float32)).clamp(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.mean(tk == kc[slots]) > 0.999                           # equal except at rounding ties
    err = np.abs(torch_decode_e4m3(kc[slots]) - want_k)
    assert np.all(err <= np.maximum(np.abs(want_k) * 2.0 ** -4, 2.0 ** -10) + 1e-6)
    tv = (torch.from_numpy(bf16_to_f32(v)) / torch.tensor(v_scale)).clamp(-448, 448).to(torch.float8_e4m3fn)
    assert np.array_equal(tv.view(torch.uint8).numpy(), vc[slots])    # v is unrotated: the plain append
    untouched = np.setdiff1d(np.arange(16), slots)
    assert np.all(kc[untouched] == 0xAA)


def test_rotation_properties():
    rng = np.random.default_rng(1)
    cos, sin = oracle.yarn_table(D, 5000)
    t = 0.1 * np.log(56.0) + 1.0
    x = bf16_bits(rng.standard_normal((1, 1, D)).astype(np.float32))
    y = bf16_bits(rng.standard_normal((1, 1, D)).astype(np.float32))
    zeros = np.zeros((1, 1, D), dtype=np.uint16)

    def rot(bits, p):
        kc, vc = oracle.new_cache(1, 1, D, oracle.KV_BF16)
        out = oracle.rope_kv_append(kc, vc, bits, zeros, zeros, np.array([p], np.int32), cos, sin,
                                    np.array([0], np.int64), 1.0, 1.0)
        return bf16_to_f32(out)[0, 0].astype(np.float64)

    x0 = bf16_to_f32(x)[0, 0].astype(np.float64)
    assert np.allclose(rot(x, 0), t * x0, rtol=2.0 ** -7)             # position 0: only the temperature
    for p in (1, 77, 4095):
        assert abs(np.linalg.norm(rot(x, p)) / (t * np.linalg.norm(x0)) - 1) < 3e-3
    base = rot(x, 1000) @ rot(y, 900)
    for shift in (5, 700, 3999):                                      # q.k depends on m - n only
        assert abs(rot(x, 1000 + shift) @ rot(y, 900 + shift) - base) < 0.05 * t * t
    assert abs(rot(x, 1000) @ rot(y, 901) - base) > 1e-3              # and does depend on it


def test_negative_slots_skip_the_cache_but_not_q():
    q, k, v, pos, slots = make_inputs(seed=3)
    slots[::2] = -1
    cos, sin = oracle.yarn_table(D, 3000)
    kc, vc = oracle.new_cache(16, 2, D)
    q_out = oracle.rope_kv_append(kc, vc, q, k, v, pos, cos, sin, slots, 0.02, 0.02)
    assert np.all(q_out.reshape(len(pos), -1).any(axis=1))
    written = np.zeros(16, dtype=bool)
    written[slots[slots >= 0]] = True
    assert np.all(kc[~written] == 0xAA) and np.all(vc[~written] == 0xAA) and np.mean(kc[written] != 0xAA) > 0.9
