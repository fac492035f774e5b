// Device helpers shared by the attention kernels (decode and prefill) for gfx950: E4M3 -> bf16
// decoding, the register tiles of one 64-position step and their loads, the matrix-core operand
// slices, validity masks and the row reductions.  Everything is per wave64; see pz_attn.hip for
// how the pieces map onto the v_mfma_f32_16x16x32_bf16 operand layouts.
#ifndef PZ_ATTN_COMMON_H
#define PZ_ATTN_COMMON_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

constexpr int kMaxWaves = 8;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ unsigned as_u32(bf16x2 v) { return __builtin_bit_cast(unsigned, v); }

// two dwords holding 8 E4M3 codes -> 8 bf16 (exact)
__device__ __forceinline__ bf16x8 dequant8(unsigned w0, unsigned w1) {
    u32x4 r;
    r[0] = as_u32(__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w0, 1.0f, false));
    r[1] = as_u32(__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w0, 1.0f, true));
    r[2] = as_u32(__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w1, 1.0f, false));
    r[3] = as_u32(__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w1, 1.0f, true));
    return __builtin_bit_cast(bf16x8, r);
}

// upper halves of two fp32 -> packed bf16 pair (truncation), first value in the low half
__device__ __forceinline__ unsigned pack_hi16(float first, float second) {
    return __builtin_amdgcn_perm(__float_as_uint(second), __float_as_uint(first), 0x07060302u);
}

// What truncation to bf16 dropped from p: p - bf16_trunc(p), exact, in one v_dot2c_f32_bf16 on the
// packed pair that already holds the truncated values: (first, second) . (-1, -0) + p.  The
// constants are spelled with a -0 half so that neither is an inline constant of the instruction
// (the inline -1.0 of a packed-bf16 operand selects the other half).
__device__ __forceinline__ float residual_first(unsigned packed, float p) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, packed), __builtin_bit_cast(bf16x2, 0x8000bf80u), p,
                                           false);
}
__device__ __forceinline__ float residual_second(unsigned packed, float p) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, packed), __builtin_bit_cast(bf16x2, 0xbf808000u), p,
                                           false);
}

// max(a, b) for a, b below FLT_MAX as the median of (a, b, FLT_MAX): one v_med3_f32.  fmaxf() costs up to three
// instructions wherever the compiler cannot prove that an operand is not a signalling NaN
// (lane-swap results, loop-carried values): it first quiets each such operand.
__device__ __forceinline__ float max2(float a, float b) { return __builtin_amdgcn_fmed3f(a, b, 3.4028234663852886e38f); }

__device__ __forceinline__ float fmax3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

// Reductions over the four 16-lane rows of a wave (lanes n, n+16, n+32, n+48) without LDS:
// v_permlane16_swap(x, x) yields (rows 0,0,2,2 | rows 1,1,3,3) and v_permlane32_swap(y, y)
// yields (low half twice | high half twice), so two swaps and two max operations reduce over the rows.
__device__ __forceinline__ float rows_max(float x) {
    u32x2 a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float y = max2(__uint_as_float(a[0]), __uint_as_float(a[1]));
    u32x2 b = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
    return max2(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

__device__ __forceinline__ float bf16_round_to_f32bits(float x, uint16_t *bits) {
    unsigned u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) { *bits = (uint16_t)((u >> 16) | 0x40u); return x; }
    u += 0x7fffu + ((u >> 16) & 1u);
    *bits = (uint16_t)(u >> 16);
    return x;
}

__device__ __forceinline__ void store_out(void *out, int out_dtype, int64_t idx, float x) {
    if (out_dtype == 0) {
        reinterpret_cast<float *>(out)[idx] = x;
    } else {
        uint16_t b;
        bf16_round_to_f32bits(x, &b);
        reinterpret_cast<uint16_t *>(out)[idx] = b;
    }
}

// One step's K pieces / V pieces of a lane.  EB = bytes per cache element (1: E4M3, 2: bf16).
template <int EB>
struct KTile {
    u32x4 k[4 * EB];
};
template <int EB>
struct VTile {
    u32x4 v[4 * EB];
};

struct LaneGeom {
    int kslot, vslot;        // which of the step's pages holds this lane's K rows / V columns
    unsigned koff, voff;     // byte offset of the lane's first piece inside the page tile
};

// D = head dimension: the row pitch of a K tile.  A 128-channel head is two 64-channel halves: the pieces of
// half h lie 64 * EB bytes further along a K row and 64 * P * EB bytes further into a V tile.
template <int P, int EB, int D = 64>
__device__ __forceinline__ LaneGeom lane_geom(int lane) {
    const int t = lane & 15, kb = lane >> 4;
    LaneGeom g;
    const int krow0 = 16 * (t >> 2) + (t & 3);        // position (within the step) of K tile 0
    g.kslot = krow0 / P;
    g.koff = (unsigned)((krow0 % P) * D * EB + kb * 16 * EB);
    const int vtok0 = 16 * kb;                         // first of the lane's 16 positions
    g.vslot = vtok0 / P;
    g.voff = (unsigned)(t * P * EB + (vtok0 % P) * EB);
    return g;
}

// STREAM: the bytes are used once (single-token decode), so they are loaded with the non-temporal
// hint and do not displace anything in L2 -- worth 10 % of the decode kernel's time.  It needs
// every load instruction to cover whole cache lines: true for E4M3 tiles; a bf16 tile spreads each
// line over two instructions, and the prefill kernel re-reads K/V through L2, so both load normally.
template <bool STREAM>
__device__ __forceinline__ u32x4 load16(const uint8_t *__restrict__ p) {
    if constexpr (STREAM) return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    else return *reinterpret_cast<const u32x4 *>(p);
}

// K: tile j holds rows 16*(t/4) + 4*j + (t%4) of the step: +4 rows per j
template <int P, int EB, bool STREAM = false, int D = 64>
__device__ __forceinline__ void load_k(KTile<EB> &tile, const uint8_t *__restrict__ kpage, unsigned koff) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < EB; ++e)
            tile.k[j * EB + e] = load16<STREAM>(kpage + koff + j * (4 * D * EB) + e * 16);
}

// V: channel tile c holds channels 16*c + t: +16 rows of P elements per c
template <int P, int EB, bool STREAM = false>
__device__ __forceinline__ void load_v(VTile<EB> &tile, const uint8_t *__restrict__ vpage, unsigned voff) {
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int e = 0; e < EB; ++e)
            tile.v[c * EB + e] = load16<STREAM>(vpage + voff + c * (16 * P * EB) + e * 16);
}

// MFMA A operand of K tile j, channel half i (channels 16*kb + 8*i .. +7)
template <int EB>
__device__ __forceinline__ bf16x8 k_operand(const KTile<EB> &tile, int j, int i) {
    if constexpr (EB == 1) return dequant8(tile.k[j][2 * i], tile.k[j][2 * i + 1]);
    else return __builtin_bit_cast(bf16x8, tile.k[2 * j + i]);
}

// MFMA A operand of V channel tile c, position half s2 (positions 16*kb + 8*s2 .. +7)
template <int EB>
__device__ __forceinline__ bf16x8 v_operand(const VTile<EB> &tile, int c, int s2) {
    if constexpr (EB == 1) return dequant8(tile.v[c][2 * s2], tile.v[c][2 * s2 + 1]);
    else return __builtin_bit_cast(bf16x8, tile.v[2 * c + s2]);
}

// zero the V elements of positions whose bit in `valid` (16 bits, bit i = lane position i) is 0
template <int EB>
__device__ __forceinline__ void mask_v(VTile<EB> &tile, unsigned valid) {
#pragma unroll
    for (int y = 0; y < 4 * EB; ++y) {           // dword y of the lane's 16 positions
        unsigned m;
        if constexpr (EB == 1) {
            unsigned b = (valid >> (4 * y)) & 15u;
            m = ((b & 1u) ? 0x000000ffu : 0u) | ((b & 2u) ? 0x0000ff00u : 0u) |
                ((b & 4u) ? 0x00ff0000u : 0u) | ((b & 8u) ? 0xff000000u : 0u);
        } else {
            unsigned b = (valid >> (2 * y)) & 3u;
            m = ((b & 1u) ? 0x0000ffffu : 0u) | ((b & 2u) ? 0xffff0000u : 0u);
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) tile.v[c * EB + y / 4][y % 4] &= m;
    }
}

// 16-bit validity mask of a lane's positions [pos0, pos0 + 16) against [j0, j1)
// Device-side inputs are held to what the caller sized: a page id from the block table to the pages
// the cache has, a sequence length to what a block-table row covers.  Inputs outside these bounds are
// the caller's mistake and give meaningless rows, but no access leaves the cache or the table.
__device__ __forceinline__ int bounded_page(int id, int num_pages) { return min(max(id, 0), num_pages - 1); }
__device__ __forceinline__ int bounded_len(int L, int max_len) { return min(L, max_len); }

__device__ __forceinline__ unsigned valid_mask(int pos0, int j0, int j1) {
    int a = min(max(j0 - pos0, 0), 16), b = min(max(j1 - pos0, 0), 16);
    return ((1u << b) - 1u) & ~((1u << a) - 1u);
}

}  // namespace

#endif
