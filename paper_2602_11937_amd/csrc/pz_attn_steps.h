// One 64-position step of decode attention for one wave64 of gfx950: S^T = K Q^T, the online
// softmax of the lane's head column, O^T += V^T P^T with the softmax denominator out of the same
// matrix-core instruction.  Shared by the decode kernels; the operand layouts are described at the
// top of pz_attn.hip.
#ifndef PZ_ATTN_STEPS_H
#define PZ_ATTN_STEPS_H

#include "pz_attn_common.h"

namespace {

struct WaveState {
    float m;          // running maximum of the log2-scaled logits of this lane's head column
    f32x4 l;          // denominator share of the lane's column (P half), every element the same
    f32x4 o[4];       // O^T: channel 16*c + 4*kb + r of the lane's head column
};

// S^T tiles of one step: sacc[j][r] = raw dot product of position 16*kb + 4*j + r with head column n
template <int EB>
__device__ __forceinline__ void qk_step(const KTile<EB> &tile, const bf16x8 (&qb)[2], f32x4 (&sacc)[4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f32x4 z = {0.f, 0.f, 0.f, 0.f};
        z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k_operand<EB>(tile, j, 0), qb[0], z, 0, 0, 0);
        sacc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k_operand<EB>(tile, j, 1), qb[1], z, 0, 0, 0);
    }
}

// Online softmax of one step for the lane's head column; returns the packed P^T operands.
__device__ __forceinline__ void softmax_step(f32x4 (&sacc)[4], float sc, unsigned lo_mask, WaveState &st,
                                             u32x4 (&pw)[2]) {
    float mx = fmax3(sacc[0][0], sacc[0][1], sacc[0][2]);
    mx = fmax3(mx, sacc[0][3], sacc[1][0]);
    mx = fmax3(mx, sacc[1][1], sacc[1][2]);
    mx = fmax3(mx, sacc[1][3], sacc[2][0]);
    mx = fmax3(mx, sacc[2][1], sacc[2][2]);
    mx = fmax3(mx, sacc[2][3], sacc[3][0]);
    mx = fmax3(mx, sacc[3][1], sacc[3][2]);
    mx = fmaxf(mx, sacc[3][3]);
    mx = rows_max(mx);
    const float m_new = fmaxf(st.m, mx * sc);          // sc > 0
    // m_new is finite here: every processed step holds at least one valid position
    const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
    st.m = m_new;
    float p[16];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            p[4 * j + r] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[j][r], sc, -m_new));
    if (__any(alpha != 1.0f)) {
#pragma unroll
        for (int c = 0; c < 4; ++c) st.o[c] *= alpha;
        st.l *= alpha;
    }
    // P^T operand: head columns 0..7 take the top bf16 of p, columns 8..15 the remainder
#pragma unroll
    for (int i = 0; i < 16; i += 2) {
        float x0 = p[i] - __uint_as_float(__float_as_uint(p[i]) & lo_mask);
        float x1 = p[i + 1] - __uint_as_float(__float_as_uint(p[i + 1]) & lo_mask);
        pw[i / 8][(i % 8) / 2] = pack_hi16(x0, x1);
    }
}

// O^T += V^T P^T, and the softmax denominator by the same instruction: a 17th "channel" whose
// V row is all ones sums the very bf16 weights that multiply V, so numerator and denominator
// share their rounding (every row of that product is the same sum over the step's 64 positions).
template <int EB>
__device__ __forceinline__ void pv_step(const VTile<EB> &tile, const u32x4 (&pw)[2], WaveState &st) {
    const u32x4 ones_bits = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};       // bf16 1.0
    const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_bits);
    st.l = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, __builtin_bit_cast(bf16x8, pw[0]), st.l, 0, 0, 0);
    st.l = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, __builtin_bit_cast(bf16x8, pw[1]), st.l, 0, 0, 0);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        st.o[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(v_operand<EB>(tile, c, 0),
                                                          __builtin_bit_cast(bf16x8, pw[0]), st.o[c], 0, 0, 0);
        st.o[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(v_operand<EB>(tile, c, 1),
                                                          __builtin_bit_cast(bf16x8, pw[1]), st.o[c], 0, 0, 0);
    }
}

// x + (x of the lane 8 places away inside its row of 16 lanes), one DPP move
__device__ __forceinline__ float add_ror8(float x) {
    return x + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x128, 0xf, 0xf, true));
}

}  // namespace

#endif
