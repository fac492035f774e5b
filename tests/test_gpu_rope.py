"""GPU parity of the fused rotary (YaRN) + quantise-and-append kernel.  The kernel gets the library's
table, the oracle its own: a token whose two table rows are equal bit for bit (all but about one in a
thousand) must come out bit-exact -- q bits and cache bytes -- and a token whose rows differ (by one unit
in the last place of an entry, tests/test_rope_table.py) may differ only where that unit crosses a
rounding boundary: by one bf16 step in q, by one adjacent E4M3 code in K.  Then attention over the cache
the kernel wrote."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_11937_amd as pz
from gpu_helpers import DEV, dev_bits, to_oracle_layout
from helpers import rel_err
from workloads import bf16_bits

pytestmark = pytest.mark.gpu
D = 64


def tables(n_pos, factor=56.0):
    """(oracle cos, oracle sin, device copies of the LIBRARY's cos and sin, rows where the two agree bitwise)"""
    lcos, lsin = pz.pz_rope_yarn_table(pz.YarnParams(factor=factor), D, n_pos)
    ocos, osin = oracle.yarn_table(D, n_pos, factor=factor)
    same = np.all(lcos == ocos, axis=1) & np.all(lsin == osin, axis=1)
    return ocos, osin, torch.from_numpy(lcos).to(DEV), torch.from_numpy(lsin).to(DEV), same


def steps_apart(a, b, sign_bit):
    """Distance of two arrays of sign-magnitude codes (bf16 bits, E4M3 bytes) in representable steps."""
    def key(x):
        x = x.astype(np.int64)
        mag = x & (sign_bit - 1)
        return np.where(x & sign_bit, -mag, mag)
    return np.abs(key(a) - key(b))


@pytest.mark.parametrize("T,Hq,Hkv,P,dtype", [(1, 8, 2, 16, pz.KV_FP8), (70, 64, 8, 64, pz.KV_FP8),
                                              (133, 16, 2, 32, pz.KV_FP8), (65, 8, 2, 64, pz.KV_BF16)])
def test_rope_append_bit_exact(T, Hq, Hkv, P, dtype):
    rng = np.random.default_rng(T)
    q = bf16_bits(rng.standard_normal((T, Hq, D)).astype(np.float32))
    k = bf16_bits((rng.standard_normal((T, Hkv, D)) * 2).astype(np.float32))
    v = bf16_bits(rng.standard_normal((T, Hkv, D)).astype(np.float32))
    cos, sin, cd, sd, same = tables(140000)
    pos = rng.integers(0, 140000, T).astype(np.int32)
    pos[1::7] = rng.choice(np.nonzero(~same)[0], size=len(pos[1::7]))   # some rows where the tables differ
    num_pages = (T + 20) // P + 2
    slots = rng.permutation(num_pages * P)[:T].astype(np.int64)
    slots[3::11] = -1
    k_scale, v_scale = 9.0 / 448, 4.5 / 448
    cache = pz.PagedCache.allocate(num_pages, P, Hkv, D, dtype, DEV, fill=0xAA if dtype == pz.KV_FP8 else -21846)
    q_dev = dev_bits(q)
    q_out = torch.zeros_like(q_dev)
    pz.pz_rope_kv_append_fp8(cache, q_dev, q_out, dev_bits(k), dev_bits(v), torch.from_numpy(pos).to(DEV), cd, sd,
                             torch.from_numpy(slots).to(DEV), T, Hq, k_scale, v_scale)
    torch.cuda.synchronize()
    okc, ovc = oracle.new_cache(num_pages * P, Hkv, D, oracle.KV_FP8 if dtype == pz.KV_FP8 else oracle.KV_BF16)
    oq = oracle.rope_kv_append(okc, ovc, q, k, v, pos, cos, sin, slots, k_scale, v_scale)
    gq = q_out.cpu().numpy().view(np.uint16)
    gk, gv = to_oracle_layout(cache)
    eq = same[pos]                                     # tokens whose table rows agree bit for bit
    assert eq.sum() >= (T + 1) // 2
    assert np.array_equal(gq[eq], oq[eq]) and np.all(steps_apart(gq[~eq], oq[~eq], 0x8000) <= 1)
    assert np.array_equal(gv, ovc)                     # V is not rotated
    written = slots >= 0
    touched = np.zeros(num_pages * P, dtype=bool)
    touched[slots[written]] = True
    assert np.array_equal(gk[~touched], okc[~touched])
    assert np.array_equal(gk[slots[written & eq]], okc[slots[written & eq]])
    ws = slots[written & ~eq]
    assert np.all(steps_apart(gk[ws], okc[ws], 0x80 if dtype == pz.KV_FP8 else 0x8000) <= 1)
    # in place: q_in == q_out
    pz.pz_rope_kv_append_fp8(cache, q_dev, q_dev, dev_bits(k), dev_bits(v), torch.from_numpy(pos).to(DEV), cd, sd,
                             torch.from_numpy(slots).to(DEV), T, Hq, k_scale, v_scale)
    torch.cuda.synchronize()
    assert np.array_equal(q_dev.cpu().numpy().view(np.uint16), gq)   # in place == out of place


def test_decode_steps_with_rotary_then_attention():
    """A short decode loop: rotary+append of each new token, then attention with the rotated q."""
    B, Hq, Hkv, P, steps = 2, 16, 2, 16, 40
    rng = np.random.default_rng(5)
    cos, sin, cd, sd, _ = tables(64)
    k_scale, v_scale = 8.0 / 448, 4.5 / 448
    num_pages = B * 3
    cache = pz.PagedCache.allocate(num_pages, P, Hkv, D, pz.KV_FP8, DEV, fill=0x7F)
    okc, ovc = oracle.new_cache(num_pages * P, Hkv, D)
    bt = np.arange(num_pages, dtype=np.int32).reshape(B, 3)
    sinks = rng.standard_normal(Hq).astype(np.float32)
    for t in range(steps):
        q = bf16_bits(rng.standard_normal((B, Hq, D)).astype(np.float32))
        k = bf16_bits(rng.standard_normal((B, Hkv, D)).astype(np.float32))
        v = bf16_bits(rng.standard_normal((B, Hkv, D)).astype(np.float32))
        pos = np.full(B, t, dtype=np.int32)
        slots = bt[:, t // P].astype(np.int64) * P + t % P
        q_dev = dev_bits(q)
        pz.pz_rope_kv_append_fp8(cache, q_dev, q_dev, dev_bits(k), dev_bits(v), torch.from_numpy(pos).to(DEV), cd, sd,
                                 torch.from_numpy(slots).to(DEV), B, Hq, k_scale, v_scale)
        oq = oracle.rope_kv_append(okc, ovc, q, k, v, pos, cos, sin, slots, k_scale, v_scale)
        lens = np.full(B, t + 1, dtype=np.int32)
        out = torch.full((B, Hq, D), float("nan"), device=DEV)
        pz.pz_decode_attn(cache, q_dev, torch.from_numpy(bt).to(DEV), 3, torch.from_numpy(lens).to(DEV), B, Hq,
                          torch.from_numpy(sinks).to(DEV), 0.125, k_scale, v_scale, 0, 0, 0, None, 0, out)
        torch.cuda.synchronize()
        want = oracle.decode_attn(okc, ovc, P, oq, bt, lens, sinks, 0.125, k_scale, v_scale, 0, accum="f64")
        assert rel_err(out.cpu().numpy(), want) <= 2e-3, t
