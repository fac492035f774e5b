"""GPU parity of the max-calibration kernels against the oracle (bit-exact: max and one division)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_11937_amd as pz
from gpu_helpers import DEV, dev_bits
from workloads import bf16_bits

pytestmark = pytest.mark.gpu


def run_calibration(batches, pow2):
    amax = torch.zeros(2, dtype=torch.float32, device=DEV)
    scales = torch.full((2,), float("nan"), dtype=torch.float32, device=DEV)
    for kb, vb in batches:
        pz.pz_kv_amax_update(dev_bits(kb), dev_bits(vb), kb.size, amax)
    pz.pz_kv_scales_from_amax(amax, pow2, scales)
    torch.cuda.synchronize()
    return amax.cpu().numpy(), scales.cpu().numpy()


@pytest.mark.parametrize("n", [1, 7, 8, 9, 1000, 4096 + 5, 3 * 1024 * 1024 + 3])
def test_amax_and_scales_match_oracle(n):
    rng = np.random.default_rng(n)
    k = bf16_bits((rng.standard_normal(n) * 5).astype(np.float32))
    v = bf16_bits((rng.standard_normal(n) * 0.01).astype(np.float32))
    if n > 100:
        k[n // 3] = 0x7FC0                                          # NaN: ignored
        v[n - 1] = bf16_bits(np.float32([-0.75]))[0]                # the maximum sits in the tail, negative
    for pow2 in (False, True):
        amax, scales = run_calibration([(k, v)], pow2)
        assert amax[0] == oracle.amax_bf16(k) and amax[1] == oracle.amax_bf16(v)
        assert scales[0] == np.float32(oracle.scale_from_amax(amax[0], pow2))
        assert scales[1] == np.float32(oracle.scale_from_amax(amax[1], pow2))


def test_running_maximum_over_batches_and_neutral_scale():
    rng = np.random.default_rng(0)
    batches = [(bf16_bits((rng.standard_normal(5000) * s).astype(np.float32)),
                bf16_bits((rng.standard_normal(5000) * s * 0.1).astype(np.float32))) for s in (1.0, 7.0, 0.2)]
    amax, scales = run_calibration(batches, True)
    allk = np.concatenate([b[0] for b in batches])
    allv = np.concatenate([b[1] for b in batches])
    assert amax[0] == oracle.amax_bf16(allk) and amax[1] == oracle.amax_bf16(allv)
    assert scales[0] == np.float32(oracle.scale_from_amax(amax[0], True))
    zeros = np.zeros(64, dtype=np.uint16)
    amax, scales = run_calibration([(zeros, zeros)], False)
    assert np.all(amax == 0) and np.all(scales == 1.0)


def test_calibrated_scales_drive_the_append():
    """End to end: calibrate on the tensor, append with the result, the largest value becomes +-448."""
    rng = np.random.default_rng(1)
    Hkv, d, P, T = 2, 64, 16, 48
    k = bf16_bits(rng.standard_normal((T, Hkv, d)).astype(np.float32))
    v = bf16_bits(rng.standard_normal((T, Hkv, d)).astype(np.float32))
    _, scales = run_calibration([(k, v)], False)
    cache = pz.PagedCache.allocate(4, P, Hkv, d, pz.KV_FP8, DEV, fill=0xAA)
    slots = torch.arange(T, dtype=torch.int64, device=DEV)
    pz.pz_kv_append_fp8(cache, dev_bits(k), dev_bits(v), slots, T, float(scales[0]), float(scales[1]))
    torch.cuda.synchronize()
    kc = cache.k.permute(0, 2, 1, 3).reshape(-1, Hkv, d)[:T].cpu().numpy()
    assert (kc & 0x7F).max() == 0x7E and not np.any((kc & 0x7F) == 0x7F)
    ok, ov = oracle.new_cache(4 * P, Hkv, d)
    oracle.kv_append(ok, ov, k, v, np.arange(T), float(scales[0]), float(scales[1]))
    assert np.array_equal(cache.k.permute(0, 2, 1, 3).reshape(-1, Hkv, d).cpu().numpy(), ok)
