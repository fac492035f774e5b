// Decode attention for a head dimension of 128 on gfx950: the same operation, operand scheme and step
// arithmetic as decode_attn_kernel (pz_attn.hip; paper Section 2, "Window attention for long-context
// inference", and Section 3, "KV Quantization"), with every head treated as two halves of 64 channels.
//
// Cache layout: K [page][Hkv][P][128], V [page][Hkv][128][P].  A step is 64 positions = 8 KiB of K and
// 8 KiB of V in FP8.  The K pieces of half h lie 64 elements further along each K row, the V pieces 64
// channel rows further into the V tile, so the lane geometry of the 64-channel kernels carries over with
// the K row pitch set to 128.  S^T = K Q^T chains the products of both halves into one accumulator; the
// softmax is the same; O^T = V^T P^T feeds eight channel tiles instead of four, and the row of ones that
// yields the denominator rides along once.
//
// One launch form only: one-wave workgroups, one per (sequence, KV head, chunk group), each walking its
// chunks back to back as one online softmax (the "direct" form of decode_attn_kernel) and writing the final
// row (single pass) or one partial into the workspace row of its first chunk (split-K; the rows of its other
// chunks are marked empty).  The model the paper accelerates has 64-channel heads; this form exists so that
// the boundary takes 128-channel caches, not as a tuned path (no balanced partition, no several waves per
// item, no in-kernel append: pz_decode_attn_append appends by a launch of its own first).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pz_attn_common.h"
#include "pz_attn_steps.h"
#include "pz_internal.h"

namespace {

constexpr int D = 128;
typedef WaveStateT<8> WideState;

template <int EB>
__device__ __forceinline__ void qk_wide(const KTile<EB> (&tile)[2], const bf16x8 (&qb)[4], f32x4 (&sacc)[4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k_operand<EB>(tile[h], j, 0), qb[2 * h], z, 0, 0, 0);
            z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k_operand<EB>(tile[h], j, 1), qb[2 * h + 1], z, 0, 0, 0);
        }
        sacc[j] = z;
    }
}

template <int EB>
__device__ __forceinline__ void pv_wide(const VTile<EB> (&tile)[2], const u32x4 (&pw)[2], WideState &st) {
    const u32x4 ones_bits = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};       // bf16 1.0
    const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_bits);
    st.l = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, __builtin_bit_cast(bf16x8, pw[0]), st.l, 0, 0, 0);
    st.l = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, __builtin_bit_cast(bf16x8, pw[1]), st.l, 0, 0, 0);
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            st.o[4 * h + c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                v_operand<EB>(tile[h], c, 0), __builtin_bit_cast(bf16x8, pw[0]), st.o[4 * h + c], 0, 0, 0);
            st.o[4 * h + c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                v_operand<EB>(tile[h], c, 1), __builtin_bit_cast(bf16x8, pw[1]), st.o[4 * h + c], 0, 0, 0);
        }
}

template <int P, int EB>
__global__ __launch_bounds__(64, EB == 1 ? 2 : 1) void decode_attn_d128_kernel(const pz::AttnParams prm) {
    constexpr int NPS = 64 / P;                        // pages per step
    constexpr int GROUP = 64 / NPS;                    // steps whose page ids fit one register
    const int lane = threadIdx.x;
    const bool final_pass = prm.split_tokens == 0;
    // same block order as decode_attn_kernel: chunk-group-major, last group first
    const int bg = blockIdx.x % (prm.B * prm.Hkv);
    const int cgrp = (int)(gridDim.x / (prm.B * prm.Hkv)) - 1 - (int)(blockIdx.x / (prm.B * prm.Hkv));
    const int b = bg / prm.Hkv, g = bg % prm.Hkv;
    const int part = g & ((1 << prm.head_shift) - 1);
    const int G = min(prm.G, prm.G_full - part * prm.G);
    const int q_first = (g >> prm.head_shift) * prm.G_full + part * prm.G;
    if (G <= 0) return;
    const int n = lane & 15, kb = lane >> 4;
    const int head = n & 7;
    const int qh = q_first + head;                     // only meaningful when head < G

    const int32_t *bt = prm.block_table + (int64_t)b * prm.max_pages;
    const int L = bounded_len(prm.seq_lens[b], prm.max_len);
    const int lo = (prm.window > 0 && L > prm.window) ? L - prm.window : 0;
    const int a0 = lo & ~63;
    const int c_first = cgrp * prm.chunks_per_group;
    const int c_last = final_pass ? 1 : min(c_first + prm.chunks_per_group, prm.n_splits);
    int j0 = lo, j1 = L;
    if (!final_pass) {
        j0 = max(lo, a0 + c_first * prm.split_tokens);
        j1 = (int)min((int64_t)L, (int64_t)a0 + (int64_t)c_last * prm.split_tokens);
    }
    const bool empty = j0 >= j1;
    if (empty && !final_pass) return;                  // no chunk of the group holds a position: nothing is written

    WideState st;
    st.m = -INFINITY;
    st.l = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < 8; ++c) st.o[c] = f32x4{0.f, 0.f, 0.f, 0.f};

    if (!empty) {
        // Q^T operand: column n holds head n % 8 of the group (zero beyond the group size), four 32-channel pieces
        bf16x8 qb[4];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            u32x4 q0 = {0, 0, 0, 0}, q1 = {0, 0, 0, 0};
            if (head < G) {
                const uint16_t *qrow = prm.q + ((int64_t)b * prm.Hq + qh) * D + 64 * h + 16 * kb;
                q0 = *reinterpret_cast<const u32x4 *>(qrow);
                q1 = *reinterpret_cast<const u32x4 *>(qrow + 8);
            }
            qb[2 * h] = __builtin_bit_cast(bf16x8, q0);
            qb[2 * h + 1] = __builtin_bit_cast(bf16x8, q1);
        }
        const unsigned lo_mask = (n >= 8) ? 0xffff0000u : 0u;
        const LaneGeom geom = lane_geom<P, EB, D>(lane);
        const int64_t page_bytes = (int64_t)prm.cache_heads * P * D * EB;
        const int cache_head = g >> prm.head_shift;
        const uint8_t *kbase = prm.k + (int64_t)cache_head * P * D * EB;
        const uint8_t *vbase = prm.v + (int64_t)cache_head * P * D * EB;
        const int pmin = lo / P, pmax = (L - 1) / P;   // pages that hold attended positions
        const float sc = prm.sc;
        const int s0 = j0 >> 6, s1 = (j1 + 63) >> 6;

        KTile<EB> kt[2];
        VTile<EB> vt[2];
        for (int gs = s0; gs < s1; gs += GROUP) {
            const int ge = min(gs + GROUP, s1);
            const int pbase = gs * NPS;
            const int ids = bounded_page(bt[min(max(pbase + lane, pmin), pmax)], prm.num_pages);
            auto page_id = [&](int idx) -> int {       // idx: page index relative to pbase, < 64
                if constexpr (NPS == 1) return __builtin_amdgcn_readlane(ids, idx);
                else return __shfl(ids, idx);
            };
            auto fetch_k = [&](int s) {
                const uint8_t *page = kbase + (int64_t)page_id(s * NPS + geom.kslot - pbase) * page_bytes;
#pragma unroll
                for (int h = 0; h < 2; ++h) load_k<P, EB, EB == 1, D>(kt[h], page + h * (64 * EB), geom.koff);
            };
            auto fetch_v = [&](int s) {
                const uint8_t *page = vbase + (int64_t)page_id(s * NPS + geom.vslot - pbase) * page_bytes;
#pragma unroll
                for (int h = 0; h < 2; ++h) load_v<P, EB, EB == 1>(vt[h], page + h * (64 * P * EB), geom.voff);
            };
            auto step = [&](int s, bool prefetch) {
                const int base = s << 6;
                const bool full = base >= j0 && base + 64 <= j1;
                const unsigned valid = full ? 0xffffu : valid_mask(base + 16 * kb, j0, j1);
                f32x4 sacc[4];
                qk_wide<EB>(kt, qb, sacc);
                if (prefetch) fetch_k(s + 1);
                if (!full) {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            sacc[j][r] = ((valid >> (4 * j + r)) & 1u) ? sacc[j][r] : -INFINITY;
                }
                u32x4 pw[2];
                softmax_step(sacc, sc, lo_mask, st, pw);
                if (!full) {
                    mask_v<EB>(vt[0], valid);
                    mask_v<EB>(vt[1], valid);
                }
                pv_wide<EB>(vt, pw, st);
                if (prefetch) fetch_v(s + 1);
            };
            fetch_k(gs);
            fetch_v(gs);
            for (int s = gs; s + 1 < ge; ++s) step(s, true);
            step(ge - 1, false);
        }
    }

    // the two P halves (columns n and n + 8) are added; columns 0..7 of the group's heads write
    const float l = add_ror8(st.l[0]);
    float scale = 1.0f;
    if (final_pass) {
        const float sink2 = (prm.sinks != nullptr && head < G) ? prm.sinks[qh] * kLog2e : -INFINITY;
        const float M = fmaxf(st.m, sink2);
        const float f = (st.m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(st.m - M);
        const float den = l * f + ((sink2 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(sink2 - M));
        scale = (den > 0.f) ? prm.v_scale * f / den : 0.f;
    }
    const bool writer = n < 8 && head < G;
    const int64_t row = ((int64_t)b * prm.Hq + qh) * prm.n_splits + c_first;      // split-K: the run's first chunk
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        f32x4 x;
#pragma unroll
        for (int r = 0; r < 4; ++r) x[r] = add_ror8(st.o[c][r]) * scale;
        if (!writer) continue;
        if (final_pass) {
            const int64_t at = ((int64_t)b * prm.Hq + qh) * D + 16 * c + 4 * kb;
            if (prm.out_dtype == 0) {
                *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(prm.out) + at) = x;
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) store_out(prm.out, 1, at + r, x[r]);
            }
        } else {
            __builtin_nontemporal_store(x, reinterpret_cast<f32x4 *>(prm.ws_acc + row * D + 16 * c + 4 * kb));
        }
    }
    if (final_pass) return;
    if (writer && kb == 0) {
        __builtin_nontemporal_store(st.m * kLn2, prm.ws_ml + row * 2);
        __builtin_nontemporal_store(l, prm.ws_ml + row * 2 + 1);
    }
    // the group's other chunks that hold positions: empty rows
    const int c_end = min(c_last, (j1 - 1 - a0) / prm.split_tokens + 1);
    const int n_rest = (c_end - c_first - 1) * G;
    for (int r = lane; r < n_rest; r += 64) {
        const int cl = 1 + r / G, h = r % G;
        const int64_t rr = ((int64_t)b * prm.Hq + q_first + h) * prm.n_splits + c_first + cl;
        __builtin_nontemporal_store(-INFINITY, prm.ws_ml + rr * 2);
        __builtin_nontemporal_store(0.0f, prm.ws_ml + rr * 2 + 1);
    }
}

}  // namespace

namespace pz {

hipError_t launch_decode_attn_d128(const AttnParams &prm, int page_size, int elem_bytes, hipStream_t stream) {
    const int n_chunks = prm.split_tokens > 0 ? prm.n_splits : 1;
    const int n_groups = (n_chunks + prm.chunks_per_group - 1) / prm.chunks_per_group;
    const dim3 grid((unsigned)(prm.B * prm.Hkv * n_groups)), block(64);
#define PZ_LAUNCH(P, EB) return launch(decode_attn_d128_kernel<P, EB>, grid, block, 0, stream, prm)
    if (elem_bytes == 1) {
        if (page_size == 64) PZ_LAUNCH(64, 1);
        if (page_size == 32) PZ_LAUNCH(32, 1);
        PZ_LAUNCH(16, 1);
    }
    if (page_size == 64) PZ_LAUNCH(64, 2);
    if (page_size == 32) PZ_LAUNCH(32, 2);
    PZ_LAUNCH(16, 2);
#undef PZ_LAUNCH
}

}  // namespace pz
