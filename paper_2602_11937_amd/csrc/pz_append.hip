// Quantise-and-append kernel for gfx950: new K/V rows (bf16) -> paged cache (E4M3 or bf16).
//
// Operation: code = e4m3(x / scale), round to nearest even, saturating at +-448 (paper
// Section 3, "KV Quantization": FP8 KV cache with max-calibrated per-layer K and V scales); the
// arithmetic of one value is in pz_quant.h.
//
// Three launch forms, the same bytes:
//   tile form (large appends: cache builds, prompts): one workgroup = up to 64 tokens of one KV head.
//     K ([page][head][P][d]): 4 threads per token, 16 channels each -> one 16-byte store; the 16
//       tokens of a wave write 16 x 64 B rows (contiguous when their slots are).
//     V ([page][head][d][P]): lane = token, each wave walks 16 channels -> byte stores that are
//       contiguous across the lanes of a wave when the tokens' slots are contiguous.
//   token form (decode-sized appends): one wave per (token, KV head), lane = channel.
//   last-token form (split-K calls of pz_decode_attn_append): as the token form, placed from the block
//     table and the sequence lengths instead of a slot mapping.
// Tokens whose slot (or page) lies outside the cache are skipped in every form.  A head dimension of 128
// ([page][head][P][128] / [page][head][128][P]) runs every form once per 64-channel half (grid z).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pz.h"
#include "pz_internal.h"
#include "pz_quant.h"

namespace {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

template <int EB>
__global__ __launch_bounds__(256) void kv_append_kernel(const pz::AppendParams prm) {
    const int64_t t0 = (int64_t)blockIdx.x * 64;
    const int g = blockIdx.y;
    const int P = prm.P, Hkv = prm.Hkv;
    const int D = prm.D, c_half = 64 * blockIdx.z;     // this workgroup's 64 channels

    {   // ---- K: thread = (token, 16-channel part)
        const int64_t t = t0 + (threadIdx.x >> 2);
        const int part = threadIdx.x & 3;
        if (t < prm.T) {
            // the row is fetched beside the slot, not after it: one memory round trip, not two
            const u32x4 *src = reinterpret_cast<const u32x4 *>(prm.k_new + (t * Hkv + g) * D + c_half + part * 16);
            const u32x4 x0 = src[0], x1 = src[1];
            const int64_t slot = prm.slot_mapping[t];
            if (slot >= 0 && slot < prm.num_slots) {
                const int64_t page = slot / P, off = slot % P;
                uint8_t *dst = prm.k + (((page * Hkv + g) * P + off) * D + c_half + part * 16) * EB;
                if constexpr (EB == 1) {
                    u32x4 o;
                    o[0] = quant4(x0[0], x0[1], prm.k_scale);
                    o[1] = quant4(x0[2], x0[3], prm.k_scale);
                    o[2] = quant4(x1[0], x1[1], prm.k_scale);
                    o[3] = quant4(x1[2], x1[3], prm.k_scale);
                    *reinterpret_cast<u32x4 *>(dst) = o;
                } else {
                    reinterpret_cast<u32x4 *>(dst)[0] = x0;
                    reinterpret_cast<u32x4 *>(dst)[1] = x1;
                }
            }
        }
    }
    {   // ---- V: lane = token, wave = 16-channel part
        const int64_t t = t0 + (threadIdx.x & 63);
        const int c0 = c_half + (threadIdx.x >> 6) * 16;
        if (t < prm.T) {
            const uint16_t *src = prm.v_new + (t * Hkv + g) * D + c0;
            // plain loads: the four waves of a workgroup read neighbouring 32-byte pieces of the same rows,
            // which only the caches turn into whole-line traffic (a streaming hint cost 45 % here)
            const u32x4 x0 = reinterpret_cast<const u32x4 *>(src)[0];
            const u32x4 x1 = reinterpret_cast<const u32x4 *>(src)[1];
            const int64_t slot = prm.slot_mapping[t];
            if (slot >= 0 && slot < prm.num_slots) {
                const int64_t page = slot / P, off = slot % P;
                uint8_t *dst = prm.v + (((page * Hkv + g) * D + c0) * P + off) * EB;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const unsigned w = (i < 8) ? x0[i / 2] : x1[(i - 8) / 2];
                    const unsigned bits = (i & 1) ? (w >> 16) : (w & 0xffffu);
                    if constexpr (EB == 1) dst[(int64_t)i * P] = (uint8_t)quant_one(bits, prm.v_scale);
                    else reinterpret_cast<uint16_t *>(dst)[(int64_t)i * P] = (uint16_t)bits;
                }
            }
        }
    }
}

// One token's row of one KV head, lane = channel c.  K: the wave writes the token's 64 contiguous
// elements; V: 64 stores a page row apart.
template <int EB>
__device__ __forceinline__ void put_token(const pz::AppendParams &prm, int64_t page, int off, int g, int c,
                                          unsigned kb16, unsigned vb16) {
    const int P = prm.P, Hkv = prm.Hkv, D = prm.D;
    uint8_t *kd = prm.k + (((page * Hkv + g) * P + off) * D + c) * EB;
    uint8_t *vd = prm.v + (((page * Hkv + g) * D + c) * P + off) * EB;
    if constexpr (EB == 1) {
        *kd = (uint8_t)quant_one(kb16, prm.k_scale);
        *vd = (uint8_t)quant_one(vb16, prm.v_scale);
    } else {
        *reinterpret_cast<uint16_t *>(kd) = (uint16_t)kb16;
        *reinterpret_cast<uint16_t *>(vd) = (uint16_t)vb16;
    }
}

// Decode-sized appends (a token or a few hundred): one wave per (token, KV head), so that the launch
// spreads over the chip instead of 64-token tiles over a few workgroups.
template <int EB>
__global__ __launch_bounds__(64) void kv_append_token_kernel(const pz::AppendParams prm) {
    const int64_t t = blockIdx.x;
    const int g = blockIdx.y, c = 64 * blockIdx.z + threadIdx.x;
    const int64_t src = (t * prm.Hkv + g) * prm.D + c;
    const unsigned kb16 = prm.k_new[src], vb16 = prm.v_new[src];
    const int64_t slot = prm.slot_mapping[t];
    if (slot < 0 || slot >= prm.num_slots) return;
    put_token<EB>(prm, slot / prm.P, (int)(slot % prm.P), g, c, kb16, vb16);
}

// The newest token of every sequence, placed from the block table and the lengths (no slot mapping):
// position L_b - 1 of sequence b.  One wave per (sequence, KV head).
template <int EB>
__global__ __launch_bounds__(64) void kv_append_last_kernel(const pz::AppendParams prm,
                                                            const int32_t *__restrict__ block_table, int max_pages,
                                                            const int32_t *__restrict__ seq_lens) {
    const int b = blockIdx.x, g = blockIdx.y, c = 64 * blockIdx.z + threadIdx.x;
    const int L = seq_lens[b];
    const int64_t src = ((int64_t)b * prm.Hkv + g) * prm.D + c;
    const unsigned kb16 = prm.k_new[src], vb16 = prm.v_new[src];
    if (L <= 0 || L > max_pages * prm.P) return;           // no token, or a length the table row does not cover
    const int pos = L - 1;
    const int page = block_table[(int64_t)b * max_pages + pos / prm.P];
    if (page < 0 || (int64_t)page * prm.P >= prm.num_slots) return;
    put_token<EB>(prm, page, pos % prm.P, g, c, kb16, vb16);
}

}  // namespace

namespace pz {

hipError_t launch_kv_append_last(const AppendParams &prm, const int32_t *block_table, int max_pages,
                                 const int32_t *seq_lens, int batch, int elem_bytes, hipStream_t stream) {
    const dim3 grid((unsigned)batch, (unsigned)prm.Hkv, (unsigned)(prm.D / 64)), block(64);
    if (elem_bytes == 1) return launch(kv_append_last_kernel<1>, grid, block, 0, stream, prm, block_table, max_pages, seq_lens);
    return launch(kv_append_last_kernel<2>, grid, block, 0, stream, prm, block_table, max_pages, seq_lens);
}

hipError_t launch_kv_append(const AppendParams &prm, int elem_bytes, hipStream_t stream) {
    // up to two waves per SIMD: the token-per-wave form (the append-form override forces one, for tests)
    const int form = launch_override(PZ_OVERRIDE_APPEND_FORM);
    const bool token_form = form >= 0 ? form == 1 : prm.T * prm.Hkv <= 8192;
    if (token_form && prm.T <= 0x7fffffff) {
        const dim3 grid((unsigned)prm.T, (unsigned)prm.Hkv, (unsigned)(prm.D / 64)), block(64);
        if (elem_bytes == 1) return launch(kv_append_token_kernel<1>, grid, block, 0, stream, prm);
        return launch(kv_append_token_kernel<2>, grid, block, 0, stream, prm);
    }
    const dim3 grid((unsigned)((prm.T + 63) / 64), (unsigned)prm.Hkv, (unsigned)(prm.D / 64)), block(256);
    if (elem_bytes == 1) return launch(kv_append_kernel<1>, grid, block, 0, stream, prm);
    return launch(kv_append_kernel<2>, grid, block, 0, stream, prm);
}

}  // namespace pz
