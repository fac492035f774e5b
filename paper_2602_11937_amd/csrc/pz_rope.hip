// Fused rotary embedding (YaRN-scaled) + quantise-and-append for gfx950.
//
// Operation: the new token's q and k are rotated by position-dependent angles before k is
// quantised into the cache; v is appended unrotated.  The paper keeps the parent model's YaRN
// positional encoding and raises its scaling factor from 32 to 56 (Section 2, "Window attention
// for long-context inference", last paragraph); the angles themselves follow the published YaRN
// rule: per frequency, blend position interpolation (frequency / factor) and extrapolation
// (frequency unchanged) with a linear ramp between the dimensions that complete beta_fast and
// beta_slow rotations over the original context, and scale cos/sin by 0.1 ln(factor) + 1.
//
// The cos/sin tables are inputs of the kernel ([n_pos][32] fp32, temperature folded in), so the
// kernel holds no transcendental: with c = cos[pos][i], s = sin[pos][i], x1 = x[i], x2 = x[i+32]
//     o[i]    = fma(x1, c, -(x2 * s))         o[i+32] = fma(x2, c, x1 * s)
// (each product rounded once, each fma rounded once -- the oracle does exactly the same).
// k: code = e4m3(o / k_scale) straight from the fp32 value; q: bf16 round-to-nearest-even of o.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pz_internal.h"
#include "pz_quant.h"

namespace {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

__device__ __forceinline__ float bf16_lo(unsigned w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ unsigned bf16_rne(float x) {
    unsigned u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// rotate the 8 channel pairs (i, i+32), i = 8*part .. 8*part+7, of one 64-channel bf16 row
__device__ __forceinline__ void rotate8(const uint16_t *row, const float *cs, const float *sn, int part,
                                        float (&o1)[8], float (&o2)[8]) {
    const u32x4 a = *reinterpret_cast<const u32x4 *>(row + 8 * part);
    const u32x4 b = *reinterpret_cast<const u32x4 *>(row + 32 + 8 * part);
    const float4 c0 = *reinterpret_cast<const float4 *>(cs + 8 * part), c1 = *reinterpret_cast<const float4 *>(cs + 8 * part + 4);
    const float4 s0 = *reinterpret_cast<const float4 *>(sn + 8 * part), s1 = *reinterpret_cast<const float4 *>(sn + 8 * part + 4);
    const float c[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
    const float s[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float x1 = (e & 1) ? bf16_hi(a[e / 2]) : bf16_lo(a[e / 2]);
        const float x2 = (e & 1) ? bf16_hi(b[e / 2]) : bf16_lo(b[e / 2]);
        o1[e] = __builtin_fmaf(x1, c[e], -__fmul_rn(x2, s[e]));
        o2[e] = __builtin_fmaf(x2, c[e], __fmul_rn(x1, s[e]));
    }
}

template <int EB>
__global__ __launch_bounds__(256) void rope_kv_append_kernel(const pz::RopeAppendParams prm) {
    const int64_t t0 = (int64_t)blockIdx.x * 64;
    const int P = prm.ap.P, Hkv = prm.ap.Hkv;
    const int64_t t = t0 + (threadIdx.x >> 2);
    const int part = threadIdx.x & 3;

    if ((int)blockIdx.y >= Hkv) {                      // ---- q head: rotate, write bf16
        const int h = blockIdx.y - Hkv;
        if (t < prm.ap.T) {
            const int pos = prm.positions[t];
            float o1[8], o2[8];
            rotate8(prm.q_in + (t * prm.Hq + h) * 64, prm.cos_tab + (int64_t)pos * 32, prm.sin_tab + (int64_t)pos * 32,
                    part, o1, o2);
            u32x4 w1, w2;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                w1[e] = bf16_rne(o1[2 * e]) | (bf16_rne(o1[2 * e + 1]) << 16);
                w2[e] = bf16_rne(o2[2 * e]) | (bf16_rne(o2[2 * e + 1]) << 16);
            }
            uint16_t *dst = prm.q_out + (t * prm.Hq + h) * 64;
            *reinterpret_cast<u32x4 *>(dst + 8 * part) = w1;
            *reinterpret_cast<u32x4 *>(dst + 32 + 8 * part) = w2;
        }
        return;
    }

    const int g = blockIdx.y;
    {   // ---- K: thread = (token, 8 channel pairs): rotate, quantise, two 8-byte stores
        if (t < prm.ap.T) {
            const int pos = prm.positions[t];
            float o1[8], o2[8];
            rotate8(prm.ap.k_new + (t * Hkv + g) * 64, prm.cos_tab + (int64_t)pos * 32, prm.sin_tab + (int64_t)pos * 32,
                    part, o1, o2);
            const int64_t slot = prm.ap.slot_mapping[t];
            if (slot >= 0 && slot < prm.ap.num_slots) {
                const int64_t page = slot / P, off = slot % P;
                uint8_t *dst = prm.ap.k + (((page * Hkv + g) * P + off) * 64) * EB;
                if constexpr (EB == 1) {
                    u32x2 w1, w2;
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        unsigned x = (unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(scaled_clamped(o1[4 * e], prm.ap.k_scale),
                                                                               scaled_clamped(o1[4 * e + 1], prm.ap.k_scale), 0, false);
                        w1[e] = (unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(scaled_clamped(o1[4 * e + 2], prm.ap.k_scale),
                                                                          scaled_clamped(o1[4 * e + 3], prm.ap.k_scale), (int)x, true);
                        unsigned y = (unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(scaled_clamped(o2[4 * e], prm.ap.k_scale),
                                                                               scaled_clamped(o2[4 * e + 1], prm.ap.k_scale), 0, false);
                        w2[e] = (unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(scaled_clamped(o2[4 * e + 2], prm.ap.k_scale),
                                                                          scaled_clamped(o2[4 * e + 3], prm.ap.k_scale), (int)y, true);
                    }
                    *reinterpret_cast<u32x2 *>(dst + 8 * part) = w1;
                    *reinterpret_cast<u32x2 *>(dst + 32 + 8 * part) = w2;
                } else {
                    u32x4 w1, w2;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        w1[e] = bf16_rne(o1[2 * e]) | (bf16_rne(o1[2 * e + 1]) << 16);
                        w2[e] = bf16_rne(o2[2 * e]) | (bf16_rne(o2[2 * e + 1]) << 16);
                    }
                    *reinterpret_cast<u32x4 *>(dst + 16 * part) = w1;
                    *reinterpret_cast<u32x4 *>(dst + 64 + 16 * part) = w2;
                }
            }
        }
    }
    {   // ---- V: lane = token, wave = 16-channel part (unrotated, as in the plain append)
        const int64_t tv = t0 + (threadIdx.x & 63);
        const int c0 = (threadIdx.x >> 6) * 16;
        if (tv < prm.ap.T) {
            const uint16_t *src = prm.ap.v_new + (tv * Hkv + g) * 64 + c0;
            const u32x4 x0 = reinterpret_cast<const u32x4 *>(src)[0];
            const u32x4 x1 = reinterpret_cast<const u32x4 *>(src)[1];
            const int64_t slot = prm.ap.slot_mapping[tv];
            if (slot >= 0 && slot < prm.ap.num_slots) {
                const int64_t page = slot / P, off = slot % P;
                uint8_t *dst = prm.ap.v + (((page * Hkv + g) * 64 + c0) * P + off) * EB;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const unsigned w = (i < 8) ? x0[i / 2] : x1[(i - 8) / 2];
                    const unsigned bits = (i & 1) ? (w >> 16) : (w & 0xffffu);
                    if constexpr (EB == 1) {
                        const float a = scaled_clamped(__uint_as_float(bits << 16), prm.ap.v_scale);
                        dst[(int64_t)i * P] = (uint8_t)((unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(a, a, 0, false) & 0xffu);
                    } else {
                        reinterpret_cast<uint16_t *>(dst)[(int64_t)i * P] = (uint16_t)bits;
                    }
                }
            }
        }
    }
}

}  // namespace

namespace pz {

hipError_t launch_rope_kv_append(const RopeAppendParams &prm, int elem_bytes, hipStream_t stream) {
    const dim3 grid((unsigned)((prm.ap.T + 63) / 64), (unsigned)(prm.ap.Hkv + prm.Hq)), block(256);
    if (elem_bytes == 1) return launch(rope_kv_append_kernel<1>, grid, block, 0, stream, prm);
    return launch(rope_kv_append_kernel<2>, grid, block, 0, stream, prm);
}

}  // namespace pz
