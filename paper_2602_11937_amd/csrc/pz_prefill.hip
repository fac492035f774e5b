// Multi-token (prefill / chunked-prefill) attention over the paged FP8 / bf16 KV cache for gfx950:
// the n newest positions of every sequence are queries, each attending causally (and inside the
// layer's sliding window, "the most recent W tokens", paper Section 2) to the cache, which already
// holds their own K/V; sinks as in the decode kernel.  This is the input half of the paper's
// 64K-input / 64K-output serving scenario.
//
// Same operand scheme as the decode kernel (pz_attn.hip): S^T = K Q^T and O^T = V^T P^T on
// v_mfma_f32_16x16x32_bf16 with K and V fed straight from 16-byte loads.  The difference is what
// the 16 columns of a column tile hold: two query TOKENS x the group's 8 heads (not one token
// twice), and one wave carries NT such tiles (2*NT query tokens), so a loaded step of K/V is used
// 2*NT times.  With no spare columns the two bf16 terms of P go through two products into the
// same accumulator.  One wave walks the whole attended range of its tokens: no split-K.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pz_attn_common.h"
#include "pz_internal.h"

namespace {

// Two waves per SIMD is the register budget (256 per lane): stating it keeps every matrix-core
// accumulator in the ordinary vector registers.  Without the bound the compiler parks accumulators
// in the accumulation registers and copies each one back before the softmax reads it (72 extra
// VALU instructions per 64-position step in a kernel whose VALUs are the bottleneck).
template <int P, int EB, int NT>
__global__ __launch_bounds__(64, 2) void prefill_attn_kernel(const pz::PrefillParams prm) {
    constexpr int NPS = 64 / P;
    constexpr int GROUP = 64 / NPS;                    // steps whose page ids fit one register
    constexpr int QT = 2 * NT;                         // query tokens per wave
    const int lane = threadIdx.x;
    const int n = lane & 15, kb = lane >> 4;
    const int head = n & 7, tok_in_tile = n >> 3;
    const int g = blockIdx.x % prm.Hkv;                // KV head fastest: tiles of a head share an XCD's L2
    const int tile = (blockIdx.x / prm.Hkv) % prm.tiles_per_seq;
    const int b = blockIdx.x / (prm.Hkv * prm.tiles_per_seq);
    // heads of this virtual KV head: a group above 8 is cut into parts of prm.G heads, the last part may be
    // smaller (or empty: then there is nothing to do)
    const int part = g & ((1 << prm.head_shift) - 1);
    const int G = min(prm.G, prm.G_full - part * prm.G);
    const int q_first = (g >> prm.head_shift) * prm.G_full + part * prm.G;   // first query head of the part
    if (G <= 0) return;

    const int q0 = prm.q_start[b], n_new = prm.q_start[b + 1] - q0;
    const int i0 = tile * QT;
    if (i0 >= n_new) return;
    const int L = bounded_len(prm.seq_lens[b], prm.max_len);
    const int W = prm.window;

    // this lane's column in column tile u: query token i0 + 2u + (n >> 3), head n & 7
    int p_col[NT], lo_col[NT];
    bool live[NT];
    bf16x8 qb[NT][2];
#pragma unroll
    for (int u = 0; u < NT; ++u) {
        const int i = i0 + 2 * u + tok_in_tile;
        live[u] = i < n_new && head < G;
        p_col[u] = L - n_new + i;                      // position of the query token
        lo_col[u] = (W > 0 && p_col[u] + 1 > W) ? p_col[u] + 1 - W : 0;
        u32x4 a = {0, 0, 0, 0}, c = {0, 0, 0, 0};
        if (live[u]) {
            const uint16_t *qrow = prm.q + ((int64_t)(q0 + i) * prm.Hq + q_first + head) * 64 + 16 * kb;
            a = *reinterpret_cast<const u32x4 *>(qrow);
            c = *reinterpret_cast<const u32x4 *>(qrow + 8);
        }
        qb[u][0] = __builtin_bit_cast(bf16x8, a);
        qb[u][1] = __builtin_bit_cast(bf16x8, c);
    }
    const int i_last = min(i0 + QT, n_new) - 1;
    const int p_first = L - n_new + i0, p_last = L - n_new + i_last;
    const int j_begin = (W > 0 && p_first + 1 > W) ? p_first + 1 - W : 0;   // first attended position of the tile
    const int j_end = p_last + 1;                                           // one past the last
    const int s0 = j_begin >> 6, s1 = (j_end + 63) >> 6;

    float m[NT];
    f32x4 lsum[NT], o[NT][4];
#pragma unroll
    for (int u = 0; u < NT; ++u) {
        m[u] = -INFINITY;
        lsum[u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < 4; ++c) o[u][c] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    const LaneGeom geom = lane_geom<P, EB>(lane);
    const int64_t page_bytes = (int64_t)prm.cache_heads * P * 64 * EB;
    const uint8_t *kbase = prm.k + (int64_t)(g >> prm.head_shift) * P * 64 * EB;
    const uint8_t *vbase = prm.v + (int64_t)(g >> prm.head_shift) * P * 64 * EB;
    const int32_t *bt = prm.block_table + (int64_t)b * prm.max_pages;
    const int pmin = j_begin / P, pmax = (j_end - 1) / P;
    const float sc = prm.sc;
    const u32x4 ones_bits = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};       // bf16 1.0
    const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_bits);

    KTile<EB> kt;
    VTile<EB> vt;
    for (int gs = s0; gs < s1; gs += GROUP) {
        const int ge = min(gs + GROUP, s1);
        const int pbase = gs * NPS;
        const int ids = bounded_page(bt[min(max(pbase + lane, pmin), pmax)], prm.num_pages);
        auto page_id = [&](int idx) -> int {
            if constexpr (NPS == 1) return __builtin_amdgcn_readlane(ids, idx);
            else return __shfl(ids, idx);
        };
        auto step = [&](int s, bool prefetch) {
            const int base = s << 6;
            const int pos0 = base + 16 * kb;           // first of the lane's 16 positions
            // K operands of the step, decoded once and used by every column tile
            bf16x8 ka[4][2];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                ka[j][0] = k_operand<EB>(kt, j, 0);
                ka[j][1] = k_operand<EB>(kt, j, 1);
            }
            if (prefetch)
                load_k<P, EB>(kt, kbase + (int64_t)page_id((s + 1) * NPS + geom.kslot - pbase) * page_bytes, geom.koff);
            // positions the cache does not hold yet (>= j_end in the last page) or that lie before
            // the tile's first attended position must not reach the products as garbage
            const bool edge = base < j_begin || base + 64 > j_end;
            if (edge) mask_v<EB>(vt, valid_mask(pos0, j_begin, j_end));
            bf16x8 va[4][2];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                va[c][0] = v_operand<EB>(vt, c, 0);
                va[c][1] = v_operand<EB>(vt, c, 1);
            }
            if (prefetch)
                load_v<P, EB>(vt, vbase + (int64_t)page_id((s + 1) * NPS + geom.vslot - pbase) * page_bytes, geom.voff);
            // the four pieces of one column tile's work on this step
            auto qk = [&](int u, f32x4 (&sacc)[4]) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    f32x4 z = {0.f, 0.f, 0.f, 0.f};
                    z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[j][0], qb[u][0], z, 0, 0, 0);
                    sacc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[j][1], qb[u][1], z, 0, 0, 0);
                }
            };
            // mask, running maximum, rescale of what is accumulated; returns the reference maximum
            auto head = [&](int u, f32x4 (&sacc)[4]) -> float {
                // causal / window mask of this lane's column (a column without a query keeps its
                // garbage: it is never written out)
                const bool col_full = !live[u] || (base >= lo_col[u] && base + 63 <= p_col[u]);
                if (!__all(col_full)) {
                    const unsigned valid = live[u] ? valid_mask(pos0, lo_col[u], p_col[u] + 1) : 0xffffu;
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            sacc[j][r] = ((valid >> (4 * j + r)) & 1u) ? sacc[j][r] : -INFINITY;
                }
                float mx = max2(sacc[0][0], sacc[0][1]);
                mx = fmax3(mx, sacc[0][2], sacc[0][3]);
#pragma unroll
                for (int j = 1; j < 4; ++j) {
                    mx = fmax3(mx, sacc[j][0], sacc[j][1]);
                    mx = fmax3(mx, sacc[j][2], sacc[j][3]);
                }
                mx = rows_max(mx);
                const float m_new = max2(m[u], mx * sc);
                // a column may have seen no attended position yet (its window starts later)
                const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
                const float alpha = __builtin_amdgcn_exp2f(m[u] - m_ref);
                m[u] = m_new;
                if (__any(alpha != 1.0f)) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) o[u][c] *= alpha;
                    lsum[u] *= alpha;
                }
                return m_ref;
            };
            auto expo = [&](const f32x4 (&sacc)[4], float m_ref, u32x4 (&ph)[2], u32x4 (&pl)[2]) {
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[i / 4][i % 4], sc, -m_ref));
                    const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[(i + 1) / 4][(i + 1) % 4], sc, -m_ref));
                    const unsigned hi = pack_hi16(p0, p1);
                    ph[i / 8][(i % 8) / 2] = hi;
                    pl[i / 8][(i % 8) / 2] = pack_hi16(residual_first(hi, p0), residual_second(hi, p1));
                }
            };
            auto pv = [&](int u, const u32x4 (&ph)[2], const u32x4 (&pl)[2]) {
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    const bf16x8 bh = __builtin_bit_cast(bf16x8, ph[s2]), bl = __builtin_bit_cast(bf16x8, pl[s2]);
                    lsum[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, bh, lsum[u], 0, 0, 0);
                    lsum[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, bl, lsum[u], 0, 0, 0);
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        o[u][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[c][s2], bh, o[u][c], 0, 0, 0);
                        o[u][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[c][s2], bl, o[u][c], 0, 0, 0);
                    }
                }
            };
#pragma unroll
            for (int u = 0; u < NT; ++u) {
                f32x4 sacc[4];
                u32x4 ph[2], pl[2];
                qk(u, sacc);
                const float m_ref = head(u, sacc);
                expo(sacc, m_ref, ph, pl);
                pv(u, ph, pl);
            }
        };
        load_k<P, EB>(kt, kbase + (int64_t)page_id(gs * NPS + geom.kslot - pbase) * page_bytes, geom.koff);
        load_v<P, EB>(vt, vbase + (int64_t)page_id(gs * NPS + geom.vslot - pbase) * page_bytes, geom.voff);
        for (int s = gs; s + 1 < ge; ++s) step(s, true);
        step(ge - 1, false);
    }

    // every lane finishes its own column: sink, normalisation, 4 x 16-byte stores
#pragma unroll
    for (int u = 0; u < NT; ++u) {
        if (!live[u]) continue;
        const int i = i0 + 2 * u + tok_in_tile;
        const int qh = q_first + head;
        const float sink2 = prm.sinks != nullptr ? prm.sinks[qh] * kLog2e : -INFINITY;
        const float M = fmaxf(m[u], sink2);
        const float f = (m[u] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m[u] - M);
        const float den = lsum[u][0] * f + ((sink2 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(sink2 - M));
        const float scale = (den > 0.f) ? prm.v_scale * f / den : 0.f;
        const int64_t at = ((int64_t)(q0 + i) * prm.Hq + qh) * 64 + 4 * kb;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            f32x4 x = o[u][c] * scale;
            if (prm.out_dtype == 0) {
                *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(prm.out) + at + 16 * c) = x;
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) store_out(prm.out, 1, at + 16 * c + r, x[r]);
            }
        }
    }
}

}  // namespace

namespace pz {

hipError_t launch_prefill_attn(const PrefillParams &prm, int page_size, int elem_bytes, int n_tiles,
                               hipStream_t stream) {
    const dim3 grid((unsigned)(prm.B * prm.tiles_per_seq * prm.Hkv)), block(64);
    (void)n_tiles;
#define PZ_LAUNCH(P, EB) return launch(prefill_attn_kernel<P, EB, PZ_PREFILL_NT>, grid, block, 0, stream, prm)
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
