"""Pins of the oracle's E4M3 codec, bf16 helpers and scale rounding (CPU only).

Nothing here re-types the oracle's formulas: the decode table is checked against PyTorch's
float8_e4m3fn (a library routine) and against the integer form (8+m)*2^(e-10) evaluated with
exact fractions; the encoder against a nearest-value search over the 127 finite magnitudes in
exact rational arithmetic, with ties to the even code.  Format facts (max finite 448, no
infinities, NaN = S.1111.111, bias 7, subnormal step 2^-9) are those of the OCP FP8 E4M3
specification, the FP8 format of the KV cache (paper Section 3, "KV Quantization").
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from helpers import division_sensitive_inputs
from workloads import bf16_bits, bf16_to_f32

ALL_CODES = np.arange(256, dtype=np.uint8)


def exact_value(code: int):
    """E4M3 value of a code as an exact Fraction (None for NaN), integer form."""
    s, e, m = code >> 7, (code >> 3) & 15, code & 7
    if e == 15 and m == 7:
        return None
    mag = Fraction(m, 512) if e == 0 else Fraction(8 + m) * Fraction(2) ** (e - 10)
    return -mag if s else mag


FINITE_POS = [(c, exact_value(c)) for c in range(0x7F)]      # codes 0x00..0x7E, ascending


def nearest_code(x: float) -> int:
    """Round-to-nearest-even E4M3 code of a finite or infinite float, saturating at 448."""
    sign = 0x80 if np.signbit(x) else 0
    if np.isinf(x):
        return sign | 0x7E
    a = abs(Fraction(float(x)))
    if a > 448:
        return sign | 0x7E
    best, best_err = None, None
    for c, val in FINITE_POS:
        err = abs(val - a)
        if best is None or err < best_err or (err == best_err and c % 2 == 0 and best % 2 == 1):
            best, best_err = c, err
    return sign | best


def test_decode_table_matches_exact_and_torch():
    dec = oracle.e4m3_decode(ALL_CODES)
    t = torch.from_numpy(ALL_CODES.copy()).view(torch.float8_e4m3fn).float().numpy()
    for c in range(256):
        ev = exact_value(c)
        if ev is None:
            assert np.isnan(dec[c]) and np.isnan(t[c])
        else:
            assert Fraction(float(dec[c])) == ev, hex(c)
            assert dec[c] == t[c]
            assert np.signbit(dec[c]) == bool(c >> 7)


def test_decode_spot_values_and_structure():
    d = oracle.e4m3_decode(ALL_CODES)
    assert d[0x7E] == 448.0 and d[0x38] == 1.0 and d[0x01] == 2.0 ** -9 and d[0x08] == 2.0 ** -6
    assert d[0x00] == 0.0 and d[0x80] == 0.0 and np.signbit(d[0x80])
    assert np.isnan(d[0x7F]) and np.isnan(d[0xFF])
    assert np.all(np.diff(d[:0x7F]) > 0)                       # strictly monotone 0x00..0x7E
    assert np.array_equal(d[0x80:0xFF], -d[0x00:0x7F])         # sign symmetry
    assert not np.any(np.isinf(d))


def test_encode_roundtrip_all_codes():
    d = oracle.e4m3_decode(ALL_CODES)
    ok = ~np.isnan(d)
    assert np.array_equal(oracle.e4m3_encode(d[ok]), ALL_CODES[ok])


def test_encode_spot_values():
    cases = [(448.0, 0x7E), (464.0, 0x7E), (1e9, 0x7E), (np.inf, 0x7E), (-np.inf, 0xFE),
             (2.0 ** -9, 0x01), (2.0 ** -10, 0x00), (1.5 * 2.0 ** -10, 0x01), (3 * 2.0 ** -10, 0x02),
             (1.0, 0x38), (-0.0, 0x80), (-2.0 ** -11, 0x80), (0.0, 0x00), (447.9, 0x7E),
             (432.0, 0x7E), (431.9, 0x7D), (416.0, 0x7D), (1.0625, 0x38), (1.1875, 0x3A),
             (0.0146484375, 0x08), (0.0166015625, 0x08), (-1.0, 0xB8), (-448.0, 0xFE)]
    for x, code in cases:
        assert int(oracle.e4m3_encode(np.float32(x))) == code, (x, hex(code))
    nan_codes = oracle.e4m3_encode(np.array([np.nan, -np.nan], dtype=np.float32))
    assert nan_codes[0] & 0x7F == 0x7F and nan_codes[1] & 0x7F == 0x7F


def test_encode_all_bf16_inputs_against_exact_search():
    bits = np.arange(65536, dtype=np.uint16)
    x = bf16_to_f32(bits)
    finite = ~np.isnan(x)
    got = oracle.e4m3_encode(x[finite])
    # values > 448 or < 2^-11 are trivially decided; run the exact search on the rest + samples
    xs = x[finite]
    want = np.empty_like(got)
    for i, v in enumerate(xs):
        a = abs(float(v))
        if a > 448:
            want[i] = (0x80 if np.signbit(v) else 0) | 0x7E
        elif a < 2.0 ** -10:
            want[i] = 0x80 if np.signbit(v) else 0
        else:
            want[i] = nearest_code(float(v))
    assert np.array_equal(got, want)


def test_encode_midpoints_and_neighbours():
    """Every midpoint between adjacent finite codes (a tie) and its fp32 neighbours."""
    vals = [float(v) for _, v in FINITE_POS]
    xs = []
    for lo, hi in zip(vals[:-1], vals[1:]):
        mid = np.float32((lo + hi) / 2)                        # exact in fp32
        xs += [mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(1e9))]
    xs += [np.float32(448), np.nextafter(np.float32(448), np.float32(1e9)), np.float32(456),
           np.float32(464), np.float32(480)]
    xs = np.array(xs, dtype=np.float32)
    xs = np.concatenate([xs, -xs])
    got = oracle.e4m3_encode(xs)
    want = np.array([nearest_code(float(v)) for v in xs], dtype=np.uint8)
    assert np.array_equal(got, want)


def test_encode_matches_torch_in_range():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * s for s in (1e-3, 0.05, 1, 30, 120)])
    x = x[np.abs(x) <= 448]
    t = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(oracle.e4m3_encode(x), t)


def test_bf16_helpers_match_torch():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(5000) * 10.0 ** rng.integers(-20, 20, 5000)).astype(np.float32)
    x = np.concatenate([x, np.float32([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38])])
    tb = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.f32_to_bf16(x), tb)
    assert np.array_equal(bf16_bits(x), tb)                    # the input generator's own rounding
    bits = np.arange(65536, dtype=np.uint16)
    ob = oracle.bf16_to_f32(bits)
    tt = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).float().numpy()
    fin = ~np.isnan(tt)                                        # NaN payloads may be quieted in transit
    assert np.array_equal(ob.view(np.uint32)[fin], tt.view(np.uint32)[fin])
    assert np.all(np.isnan(ob[~fin]))


def test_quantize_is_one_division_then_encode():
    rng = np.random.default_rng(2)
    xb = bf16_bits(rng.standard_normal(4000).astype(np.float32) * 3)
    for scale in (1.0, 0.0123, 4.8 / 448, 0.5, 2.0 ** -7, 3.0):
        got = oracle.quantize(xb, scale)
        r = (bf16_to_f32(xb).astype(np.float32) / np.float32(scale)).astype(np.float32)
        want = np.array([nearest_code(float(v)) for v in r], dtype=np.uint8)
        assert np.array_equal(got, want), scale
    assert np.array_equal(oracle.quantize(xb, 1.0), oracle.e4m3_encode(bf16_to_f32(xb)))


def test_quantize_divides_and_does_not_multiply_by_the_reciprocal():
    """x / scale and x * (1 / scale) differ by an ulp now and then, and when the quotient sits on the
    midpoint between two codes that ulp decides the code.  Such inputs are built on purpose: for a
    bf16 x and a midpoint mid, scales within a few ulps of x / mid put the quotient on or beside mid.
    The cases where numpy's IEEE fp32 division and the reciprocal product give different codes (by
    PyTorch's conversion) are kept, and the oracle must side with the division on every one."""
    found = division_sensitive_inputs()
    assert len(found) >= 50, len(found)
    for xb, sc, r1, r2 in found[:300]:
        got = int(oracle.quantize(np.array([xb], dtype=np.uint16), sc)[0])
        assert got == nearest_code(r1) and got != nearest_code(r2), (hex(xb), sc)


def test_power_of_two_scale_only_shifts_the_exponent():
    """With a power-of-two scale the rounding is that of the unscaled value: the code's exponent
    field moves by -log2(scale) and the mantissa bits are unchanged, whenever both the scaled and
    unscaled values are in the normal range (the property behind the paper's choice to round
    scales up to powers of two, Section 3 "KV Quantization")."""
    rng = np.random.default_rng(3)
    x = rng.standard_normal(6000).astype(np.float32)
    xb = bf16_bits(x)
    base = oracle.quantize(xb, 1.0)
    for k in (1, 2, 4):
        scaled = oracle.quantize(xb, 2.0 ** -k)
        e0 = (base >> 3) & 15
        a = np.abs(bf16_to_f32(xb))
        ok = (a >= 2.0 ** -6) & (a * 2.0 ** k <= 448) & (e0 + k <= 15)
        assert ok.sum() > 3000
        assert np.array_equal(scaled[ok], base[ok] + (k << 3))
        # and division by a power of two equals multiplication by its reciprocal, bit for bit
        r1 = bf16_to_f32(xb) / np.float32(2.0 ** -k)
        r2 = bf16_to_f32(xb) * np.float32(2.0 ** k)
        assert np.array_equal(r1.view(np.uint32), r2.view(np.uint32))


def test_round_scale_up_pow2():
    for s, want in [(0.3, 0.5), (0.5, 0.5), (0.51, 1.0), (4.8 / 448, 2.0 ** -6), (2.0 ** -9, 2.0 ** -9),
                    (0.0107, 2.0 ** -6), (1.0, 1.0), (0.99, 1.0)]:
        assert oracle.round_scale_up_pow2(s) == want
    rng = np.random.default_rng(4)
    for s in rng.uniform(1e-4, 1.0, 200):
        r = oracle.round_scale_up_pow2(np.float32(s))
        assert r >= np.float32(s) and r < 2 * np.float32(s) and np.log2(r) == int(np.log2(r))


def test_max_calibration_amax_and_scale():
    """amax against numpy's nanmax; the scale is the paper's max calibration (amax lands on 448)."""
    rng = np.random.default_rng(5)
    x = (rng.standard_normal(10007) * 3).astype(np.float32)
    x[17] = -41.5
    x[100] = np.nan
    bits = bf16_bits(x)
    bits[100] = 0x7FC1
    want = np.nanmax(np.abs(bf16_to_f32(bits)))
    assert oracle.amax_bf16(bits) == want == 41.5
    assert oracle.amax_bf16(np.zeros(0, dtype=np.uint16)) == 0.0
    assert oracle.amax_bf16(np.array([0x8000, 0x0000], dtype=np.uint16)) == 0.0
    s = oracle.scale_from_amax(want)
    assert s == float(np.float32(want) / np.float32(448))
    assert int(oracle.quantize(bf16_bits(np.float32([-41.5])), s)[0]) == 0xFE      # amax -> -448
    assert oracle.scale_from_amax(0.0) == 1.0 and oracle.scale_from_amax(0.0, True) == 1.0
    p2 = oracle.scale_from_amax(want, True)
    assert p2 == 0.125 and s <= p2 < 2 * s
    assert oracle.scale_from_amax(448.0 * 0.25, True) == 0.25                      # already a power of two
    # a power-of-two scale never overflows what the raw scale did not: |x / p2| <= |x / s| <= 448
    codes = oracle.quantize(np.delete(bits[:2000], 100), p2)      # without the NaN element
    assert not np.any((codes & 0x7F) == 0x7F) and (codes & 0x7F).max() <= 0x7E
