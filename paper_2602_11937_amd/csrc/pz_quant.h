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

}  // namespace

#endif
