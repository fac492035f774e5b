// E4M3 quantisation of one value for gfx950, shared by the kernels that write the cache.
//
// code = e4m3(x / scale), round to nearest even, saturating at +-448 (paper Section 3, "KV
// Quantization").  The division is a correctly rounded fp32 division; the hardware convert
// (v_cvt_pk_fp8_f32) rounds to nearest even but turns out-of-range inputs into NaN, so the quotient
// is clamped to +-448 first (NaN inputs bypass the clamp and stay NaN).
#ifndef PZ_QUANT_H
#define PZ_QUANT_H

#include <hip/hip_runtime.h>

namespace {

__device__ __forceinline__ float scaled_clamped(float x, float scale) {
    const float r = __fdiv_rn(x, scale);
    return (r != r) ? r : __builtin_amdgcn_fmed3f(r, -448.0f, 448.0f);
}

// one bf16 value (bit pattern in the low 16 bits) -> one E4M3 code
__device__ __forceinline__ unsigned quant_one(unsigned bits16, float scale) {
    const float a = scaled_clamped(__uint_as_float(bits16 << 16), scale);
    return (unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(a, a, 0, false) & 0xffu;
}

// two bf16 values packed in one dword -> two E4M3 codes in the low (hi=false) or high word of old
__device__ __forceinline__ unsigned quant_pair(unsigned packed_bf16, float scale, unsigned old, bool hi) {
    const float a = scaled_clamped(__uint_as_float(packed_bf16 << 16), scale);
    const float b = scaled_clamped(__uint_as_float(packed_bf16 & 0xffff0000u), scale);
    return hi ? (unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, (int)old, true)
              : (unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, (int)old, false);
}

// two dwords of packed bf16 pairs (4 values) -> 4 E4M3 codes in one dword, same element order
__device__ __forceinline__ unsigned quant4(unsigned p0, unsigned p1, float scale) {
    return quant_pair(p1, scale, quant_pair(p0, scale, 0u, false), true);
}

}  // namespace

#endif
