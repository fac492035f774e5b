// One 64-position step of decode attention for one wave64 of gfx950: S^T = K Q^T, the online
// softmax of the lane's head column, O^T += V^T P^T with the softmax denominator out of the same
// matrix-core instruction.  Shared by the decode kernels; the operand layouts are described at the
// top of pz_attn.hip.
#ifndef PZ_ATTN_STEPS_H
#define PZ_ATTN_STEPS_H

#include "pz_attn_common.h"
#include "pz_internal.h"
#include "pz_quant.h"

namespace {

template <int NO>
struct WaveStateT {
    float m;          // running maximum of the log2-scaled logits of this lane's head column
    f32x4 l;          // denominator share of the lane's column (P half), every element the same
    f32x4 o[NO];      // O^T: channel 16*c + 4*kb + r of the lane's head column (NO = head dimension / 16)
};
typedef WaveStateT<4> WaveState;

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
template <int NO>
__device__ __forceinline__ void softmax_step(f32x4 (&sacc)[4], float sc, unsigned lo_mask, WaveStateT<NO> &st,
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
        for (int c = 0; c < NO; ++c) st.o[c] *= alpha;
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

// ---- the newest token of a sequence, fused append (pz_decode_attn_append) --------------------------------
// The run that ends at position L - 1 does not read that position from the cache.  It walks the cached
// positions below it exactly as a call without append would, and then, behind the loop, takes the token's K
// row and V column from k_new / v_new (one load round trip together with the position's block-table
// entry), quantises them with the append kernel's arithmetic (pz_quant.h: the same codes, so the outputs
// are bit-identical to append-then-attend), attends to that one position as a last step of its own, and
// writes the cache bytes.  Everything the append adds sits behind the step loop: nothing is loaded, held or
// decided inside it (a load left pending across that loop, or a branch on the append inside it, changed the
// compiler's wait counts and loop shape and cost 4 to 8 % of the whole launch), nothing the wave reads later
// is written, and the 64 scattered V bytes leave when the wave's streaming is over.
template <int EB>
struct NewToken {
    u32x4 k[EB];      // the lane's 16 channels (16*kb ..) of the K row, as they lie in a K tile
    unsigned v[EB];   // the lane's channels 16*c + t, c = 0..3, of the V column: codes (bf16: pairs) in c order
};

// x | (x of the other lanes of the quad selected by a DPP quad permutation)
template <int CTRL>
__device__ __forceinline__ unsigned or_quad(unsigned x) {
    return x | (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, true);
}

// From the token's row with lane = channel (kbits / vbits: bf16 bit patterns of channel `lane`) to the tile
// form: one quantisation per lane and row, then the codes travel between lanes.
template <int EB>
__device__ __forceinline__ NewToken<EB> pack_new_token(unsigned kbits, unsigned vbits, float k_scale, float v_scale,
                                                       int lane) {
    const int t = lane & 15, kb = lane >> 4;
    NewToken<EB> nt;
    if constexpr (EB == 1) {
        // every lane of a quad ends up with the dword of its quad's four channels
        unsigned kq = quant_one(kbits, k_scale) << (8 * (lane & 3));
        kq = or_quad<0xB1>(kq);                        // quad_perm 1,0,3,2
        kq = or_quad<0x4E>(kq);                        // quad_perm 2,3,0,1
#pragma unroll
        for (int y = 0; y < 4; ++y) nt.k[0][y] = (unsigned)__shfl((int)kq, 16 * kb + 4 * y);
        const unsigned vq = quant_one(vbits, v_scale);
        nt.v[0] = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) nt.v[0] |= (unsigned)__shfl((int)vq, 16 * c + t) << (8 * c);
    } else {
        unsigned kp = kbits << (16 * (lane & 1));
        kp = or_quad<0xB1>(kp);                        // both lanes of a pair hold the pair's dword
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int y = 0; y < 4; ++y) nt.k[e][y] = (unsigned)__shfl((int)kp, 16 * kb + 8 * e + 2 * y);
#pragma unroll
        for (int h = 0; h < 2; ++h)
            nt.v[h] = (unsigned)__shfl((int)vbits, 32 * h + t) | ((unsigned)__shfl((int)vbits, 32 * h + 16 + t) << 16);
    }
    return nt;
}

// position r (0..63, uniform) of the step whose tiles are in kt: the lanes that hold its K row take the new row
template <int EB>
__device__ __forceinline__ void put_new_k(KTile<EB> &kt, const NewToken<EB> &nt, int lane, int r) {
    const int t = lane & 15;
    const bool mine = t == (((r >> 4) << 2) | (r & 3));      // row 16*(t/4) + 4*j + t%4 == r
    const int jr = (r >> 2) & 3;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < EB; ++e)
            if (j == jr && mine) kt.k[j * EB + e] = nt.k[e];
}

// ... and the lanes that hold its V column (positions 16*kb .. 16*kb + 15 of channels 16*c + t) the new elements
template <int EB>
__device__ __forceinline__ void put_new_v(VTile<EB> &vt, const NewToken<EB> &nt, int lane, int r) {
    const bool mine = (lane >> 4) == (r >> 4);
    if constexpr (EB == 1) {
        const int dw = (r & 15) >> 2, sh = 8 * (r & 3);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const unsigned code = (nt.v[0] >> (8 * c)) & 0xffu;
#pragma unroll
            for (int y = 0; y < 4; ++y)
                if (y == dw && mine) vt.v[c][y] = (vt.v[c][y] & ~(0xffu << sh)) | (code << sh);
        }
    } else {
        const int e_r = (r & 15) >> 3, dw = (r & 7) >> 1, sh = 16 * (r & 1);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const unsigned bits = (nt.v[c >> 1] >> (16 * (c & 1))) & 0xffffu;
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int y = 0; y < 4; ++y)
                    if (e == e_r && y == dw && mine) vt.v[c * 2 + e][y] = (vt.v[c * 2 + e][y] & ~(0xffffu << sh)) | (bits << sh);
        }
    }
}

// The newest token's cache bytes, lane = channel: the K row is one contiguous piece, the V column one element
// in each of the 64 channel rows.
template <int P, int EB>
__device__ __forceinline__ void store_new_token(const pz::AttnParams &prm, unsigned kbits, unsigned vbits, int64_t page,
                                                int off, int cache_head, int lane) {
    const int64_t tile = (page * prm.cache_heads + cache_head) * P * 64;      // elements before this (page, head)
    uint8_t *kd = prm.k + (tile + (int64_t)off * 64 + lane) * EB;
    uint8_t *vd = prm.v + (tile + (int64_t)lane * P + off) * EB;
    if constexpr (EB == 1) {
        *kd = (uint8_t)quant_one(kbits, prm.k_scale);
        *vd = (uint8_t)quant_one(vbits, prm.v_scale);
    } else {
        *reinterpret_cast<uint16_t *>(kd) = (uint16_t)kbits;
        *reinterpret_cast<uint16_t *>(vd) = (uint16_t)vbits;
    }
}

// ---- one run of steps ------------------------------------------------------------------------------------
// Steps [s0, s1) of sequence b for (virtual) KV head g, positions [j0, j1) of them attended, folded into
// `st` as one online softmax.  The steps are walked in groups whose page ids sit in two registers (lane i
// of ids0 / ids1 holds the physical page of page index pbase + i / pbase + 64 + i, clamped to attended
// pages).  Inside a group the K buffer is refilled right after QK^T has consumed it and the V buffer right
// after PV, unconditionally; the group's last step is peeled so that no load is conditional and every wait
// counts exactly the loads issued after the one needed.  use_early: early0 / early1 already hold the
// block-table entries of the first group (read before the sequence length was known).
template <int P, int EB>
__device__ __forceinline__ void run_steps(const pz::AttnParams &prm, WaveState &st, const int32_t *__restrict__ bt,
                                          int b, int g, int G, int q_first, int lane, int L, int lo, int j0, int j1,
                                          int s0, int s1, bool use_early, int early0, int early1) {
    constexpr int NPS = 64 / P;                        // pages per step
    constexpr int GROUP = 128 / NPS;                   // steps whose page ids fit two registers
    const int n = lane & 15, kb = lane >> 4;
    const int head = n & 7;
    // Q^T operand: column n holds head n%8 of the group (zero beyond the group size)
    bf16x8 qb[2];
    {
        u32x4 q0 = {0, 0, 0, 0}, q1 = {0, 0, 0, 0};
        if (head < G) {
            const uint16_t *qrow = prm.q + ((int64_t)b * prm.Hq + q_first + head) * 64 + 16 * kb;
            q0 = *reinterpret_cast<const u32x4 *>(qrow);
            q1 = *reinterpret_cast<const u32x4 *>(qrow + 8);
        }
        qb[0] = __builtin_bit_cast(bf16x8, q0);
        qb[1] = __builtin_bit_cast(bf16x8, q1);
    }
    const unsigned lo_mask = (n >= 8) ? 0xffff0000u : 0u;
    const LaneGeom geom = lane_geom<P, EB>(lane);
    const int64_t page_bytes = (int64_t)prm.cache_heads * P * 64 * EB;
    const int cache_head = g >> prm.head_shift;
    const uint8_t *kbase = prm.k + (int64_t)cache_head * P * 64 * EB;
    const uint8_t *vbase = prm.v + (int64_t)cache_head * P * 64 * EB;
    const int pmin = lo / P, pmax = (L - 1) / P;       // pages that hold attended positions
    const float sc = prm.sc;
    // fused append: this run ends at position L - 1 of a sequence whose length is what the caller gave; the
    // loop below then stops one position short (possibly a whole step, possibly with nothing left to walk)
    const bool newest = prm.k_new != nullptr && j1 == L && s1 > ((L - 1) >> 6) && prm.seq_lens[b] == L;
    if (newest) {
        j1 = L - 1;
        s1 = (j1 + 63) >> 6;
    }

    KTile<EB> kt;
    VTile<EB> vt;
    for (int gs = s0; gs < s1; gs += GROUP) {
        const int ge = min(gs + GROUP, s1);
        const int pbase = gs * NPS;
        int ids0, ids1;
        if (use_early && gs == s0) {
            const int last = pmax - pbase;             // >= 0: the group holds an attended position
            const int fix0 = __shfl(early0, min(last, 63));
            const int fix1 = __shfl(early1, min(max(last - 64, 0), 63));
            ids0 = lane <= last ? early0 : fix0;
            ids1 = last < 64 ? fix0 : (lane + 64 <= last ? early1 : fix1);
        } else {
            ids0 = bt[min(max(pbase + lane, pmin), pmax)];
            ids1 = bt[min(max(pbase + 64 + lane, pmin), pmax)];
        }
        ids0 = bounded_page(ids0, prm.num_pages);
        ids1 = bounded_page(ids1, prm.num_pages);
        auto page_id = [&](int idx) -> int {           // idx: page index relative to pbase, < 128
            if constexpr (NPS == 1) {
                const int a = __builtin_amdgcn_readlane(ids0, idx & 63);
                const int c = __builtin_amdgcn_readlane(ids1, idx & 63);
                return idx < 64 ? a : c;
            } else {
                const int a = __shfl(ids0, idx & 63), c = __shfl(ids1, idx & 63);
                return idx < 64 ? a : c;
            }
        };
        auto k_page = [&](int s) -> const uint8_t * {
            return kbase + (int64_t)page_id(s * NPS + geom.kslot - pbase) * page_bytes;
        };
        auto v_page = [&](int s) -> const uint8_t * {
            return vbase + (int64_t)page_id(s * NPS + geom.vslot - pbase) * page_bytes;
        };
        auto step = [&](int s, bool prefetch) {
            const int base = s << 6;
            const bool full = base >= j0 && base + 64 <= j1;
            const unsigned valid = full ? 0xffffu : valid_mask(base + 16 * kb, j0, j1);
            f32x4 sacc[4];
            qk_step<EB>(kt, qb, sacc);
            if (prefetch) load_k<P, EB, EB == 1>(kt, k_page(s + 1), geom.koff);
            if (!full) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        sacc[j][r] = ((valid >> (4 * j + r)) & 1u) ? sacc[j][r] : -INFINITY;
            }
            u32x4 pw[2];
            softmax_step(sacc, sc, lo_mask, st, pw);
            if (!full) mask_v<EB>(vt, valid);
            pv_step<EB>(vt, pw, st);
            if (prefetch) load_v<P, EB, EB == 1>(vt, v_page(s + 1), geom.voff);
        };
        load_k<P, EB, EB == 1>(kt, k_page(gs), geom.koff);
        load_v<P, EB, EB == 1>(vt, v_page(gs), geom.voff);
        for (int s = gs; s + 1 < ge; ++s) step(s, true);
        step(ge - 1, false);
    }

    if (newest) {
        // position L - 1 from k_new / v_new: a step of its own in which only that position is valid
        const int r = (L - 1) & 63;
        const int64_t at = ((int64_t)b * prm.cache_heads + cache_head) * 64 + lane;
        const unsigned new_k = prm.k_new[at], new_v = prm.v_new[at];   // the token's element of channel `lane`
        const int newest_page = bt[pmax];                              // as the caller gave it
        const NewToken<EB> nt = pack_new_token<EB>(new_k, new_v, prm.k_scale, prm.v_scale, lane);
#pragma unroll
        for (int i = 0; i < 4 * EB; ++i) {
            kt.k[i] = u32x4{0, 0, 0, 0};
            vt.v[i] = u32x4{0, 0, 0, 0};
        }
        put_new_k<EB>(kt, nt, lane, r);
        put_new_v<EB>(vt, nt, lane, r);
        const unsigned valid = kb == (r >> 4) ? 1u << (r & 15) : 0u;
        f32x4 sacc[4];
        qk_step<EB>(kt, qb, sacc);
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) sacc[j][i] = ((valid >> (4 * j + i)) & 1u) ? sacc[j][i] : -INFINITY;
        u32x4 pw[2];
        softmax_step(sacc, sc, lo_mask, st, pw);
        pv_step<EB>(vt, pw, st);                       // every other element of the V tile is zero
        // the token's cache bytes; several virtual heads may share a cache head: the first of them writes.  A
        // page the cache does not have: nothing is written.
        if ((g & ((1 << prm.head_shift) - 1)) == 0 && newest_page >= 0 && newest_page < prm.num_pages)
            store_new_token<P, EB>(prm, new_k, new_v, newest_page, (L - 1) % P, cache_head, lane);
    }
}

}  // namespace

#endif
