// Max calibration of the per-layer KV scales for gfx950.
//
// Operation (paper Section 3, "KV Quantization"): the K and V scales of a layer come from max
// calibration over a dataset -- scale = amax / 448 so that the largest magnitude lands on the
// largest E4M3 value -- and are then rounded up to a power of two.  The dataset is streamed in
// batches; `amax` (two floats on the device: K, V) carries the running maxima between calls.
//
// amax kernel: HBM-bound streaming read of bf16 (2 bytes per element, each read once).  The
// magnitude of a bf16 value is its low 15 bits, and for non-NaN values the order of those bit
// patterns is the order of the magnitudes, so the maximum is taken on integers; NaN elements are
// ignored.  Waves read contiguous 8 KiB tiles, 16 bytes per lane and load; at most one atomic max
// per wave.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pz_internal.h"

namespace {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

__device__ __forceinline__ unsigned mag_max2(unsigned best, unsigned packed) {
    unsigned lo = packed & 0x7fffu, hi = (packed >> 16) & 0x7fffu;
    lo = lo > 0x7f80u ? 0u : lo;                       // NaN: ignored
    hi = hi > 0x7f80u ? 0u : hi;
    return max(best, max(lo, hi));
}

// One wave per workgroup: a plain read loop measured 4 % faster with one-wave workgroups than with
// four-wave ones on this chip.  A wave owns a contiguous run of tiles and has the next tile's loads
// in flight while it reduces the current one.
__global__ __launch_bounds__(64) void kv_amax_kernel(const uint16_t *__restrict__ k,
                                                     const uint16_t *__restrict__ v, int64_t n,
                                                     int64_t tiles_per_wave, float *__restrict__ amax) {
    const uint16_t *x = blockIdx.y == 0 ? k : v;
    const int64_t n8 = n / 8;
    const u32x4 *x8 = reinterpret_cast<const u32x4 *>(x);
    unsigned best = 0;
    const int lane = threadIdx.x;
    const int64_t n_tiles = n8 / 512;                  // 512 x 16 bytes = 8 KiB
    const int64_t t_begin = min((int64_t)blockIdx.x * tiles_per_wave, n_tiles);
    const int64_t t_end = min(t_begin + tiles_per_wave, n_tiles);
    auto fetch = [&](u32x4 (&a)[8], int64_t t) {
        const u32x4 *p = x8 + t * 512 + lane;
#pragma unroll
        for (int u = 0; u < 8; ++u) a[u] = __builtin_nontemporal_load(p + u * 64);   // read once: streaming hint
    };
    auto reduce = [&](const u32x4 (&a)[8]) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int e = 0; e < 4; ++e) best = mag_max2(best, a[u][e]);
    };
    u32x4 a[8], b[8];
    if (t_begin < t_end) fetch(a, t_begin);
    for (int64_t t = t_begin; t < t_end; t += 2) {
        if (t + 1 < t_end) fetch(b, t + 1);
        reduce(a);
        if (t + 1 < t_end) {
            if (t + 2 < t_end) fetch(a, t + 2);
            reduce(b);
        }
    }
    for (int64_t i = n_tiles * 512 + (int64_t)blockIdx.x * 64 + lane; i < n8; i += (int64_t)gridDim.x * 64) {
        const u32x4 r = x8[i];                         // what does not fill a tile
#pragma unroll
        for (int e = 0; e < 4; ++e) best = mag_max2(best, r[e]);
    }
    if (blockIdx.x == 0 && lane < (int)(n - n8 * 8)) {  // tail elements
        unsigned m = x[n8 * 8 + lane] & 0x7fffu;
        best = max(best, m > 0x7f80u ? 0u : m);
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) best = max(best, (unsigned)__shfl_xor((int)best, d));
    // fp32 bit patterns of non-negative floats are ordered like the floats themselves.  The running
    // maximum only grows, so a wave whose maximum is not above a (possibly stale) read of it has
    // nothing to add; this keeps the thousands of waves from queueing on one address.
    unsigned *slot = reinterpret_cast<unsigned *>(amax) + blockIdx.y;
    if (lane == 0 && (best << 16) > __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
        atomicMax(slot, best << 16);
}

__global__ void kv_scales_kernel(const float *__restrict__ amax, int round_up_pow2, float *__restrict__ scales) {
    const int i = threadIdx.x;
    if (i >= 2) return;
    float s = __fdiv_rn(amax[i], 448.0f);
    if (!(s > 0.0f)) {
        s = 1.0f;                                      // nothing seen (or NaN): the neutral scale
    } else if (round_up_pow2 && s < INFINITY) {
        unsigned u = __float_as_uint(s);
        if (u & 0x007fffffu) {                         // not a power of two already
            if ((u >> 23) == 0) {                      // subnormal: go through a normal number
                const float t = s * 0x1p24f;
                u = (__float_as_uint(t) & 0x7f800000u) + 0x00800000u;
                s = __uint_as_float(u) * 0x1p-24f;
            } else {
                s = __uint_as_float((u & 0x7f800000u) + 0x00800000u);
            }
        }
    }
    scales[i] = s;
}

}  // namespace

namespace pz {

hipError_t launch_kv_amax(const uint16_t *k, const uint16_t *v, int64_t n, float *amax, hipStream_t stream) {
    // 8 tiles (64 KiB) per wave until the grid would pass 65536 waves per tensor
    const int64_t n_tiles = n / 8 / 512;
    int64_t per = 8;
    if ((n_tiles + per - 1) / per > 65536) per = (n_tiles + 65535) / 65536;
    int64_t blocks = (n_tiles + per - 1) / per;
    if (blocks < 1) blocks = 1;
    return launch(kv_amax_kernel, dim3((unsigned)blocks, 2), dim3(64), 0, stream, k, v, n, per, amax);
}

hipError_t launch_kv_scales(const float *amax, int round_up_pow2, float *scales, hipStream_t stream) {
    return launch(kv_scales_kernel, dim3(1), dim3(64), 0, stream, amax, round_up_pow2, scales);
}

}  // namespace pz
