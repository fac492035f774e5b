// Decode attention over the paged FP8 / bf16 KV cache for gfx950 (MI355X): split-K partial or
// single-pass kernel, and the log-sum-exp merge kernel.
//
// Operation: softmax attention of one query token per sequence against the cached K/V, grouped
// query heads sharing a KV head, optional sliding window ("most recent W tokens", paper
// Section 2, "Window attention for long-context inference"), cache stored as E4M3 codes with
// per-layer K/V scales that multiply on dequantisation (paper Section 3, "KV Quantization").
//
// Mapping to the hardware (one wave64 = one independent stream over the KV of one KV head):
//   * A "step" is 64 consecutive logical positions of one (sequence, KV head): 4 KiB of K and
//     4 KiB of V in FP8.  Every lane fetches 4 + 4 aligned 16-byte pieces straight from HBM into
//     registers; each wave-wide load instruction covers whole 256-byte (K) or 1-KiB (V) runs.
//     There is no reuse between waves, so nothing is staged through LDS; the K registers are
//     refilled with step s+1 as soon as QK^T of step s has consumed them, the V registers as
//     soon as PV of step s has, so about one step's worth of loads is always in flight.
//   * S^T = K Q^T on the matrix cores (v_mfma_f32_16x16x32_bf16): A = 16 cached positions x 32
//     channels, B = Q^T with the group's (up to 8) query heads in columns 0..7 and again in
//     columns 8..15.  E4M3 -> bf16 is exact (one v_cvt_scalef32_pk_bf16_fp8 per two codes), q is
//     bf16, products are exact in fp32.
//   * The result layout gives every lane 16 consecutive positions of one query-head column, so
//     the online softmax needs cross-lane traffic only for the running maximum (lanes n, n+16,
//     n+32, n+48).  exp is v_exp_f32 on log2-scaled logits.
//   * O^T = V^T P^T on the matrix cores with V stored channel-major ([d][page_size]), so the A
//     operand is again a direct 8-byte slice of what was loaded.  P is fed as bf16 in two
//     terms: columns 0..7 carry the top 8 significant bits of p, columns 8..15 the next 8, which
//     keeps p to ~2^-16 relative; the two halves are added at the end.  The softmax
//     denominator comes out of the same instruction: a row of ones sums the same bf16 weights.
//   * Waves of a workgroup own disjoint step ranges and are merged through LDS (2 KiB per
//     wave); the workgroup then writes either a sink-free partial (split-K) or the final row.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pz_attn_common.h"
#include "pz_attn_steps.h"
#include "pz_internal.h"
#include "pz_quant.h"

namespace {

// Grid: one workgroup per (sequence, KV head, chunk group).  Two modes:
//   n_waves == 1 ("direct"): the wave walks every chunk of its group back to back as one online
//     softmax and writes the final row (single pass) straight from registers, or (split-K) one
//     partial for the group: it goes to the workspace row of the group's first chunk, the rows of
//     its other chunks are marked empty (m = -inf, l = 0) and the merge kernel skips them.
//   n_waves  > 1: one chunk (or the whole sequence) per workgroup, its steps dealt to the waves,
//     merged through LDS.
template <int P, int EB>
__global__ __launch_bounds__(64 * kMaxWaves) void decode_attn_kernel(const pz::AttnParams prm) {
    constexpr int NPS = 64 / P;                        // pages per step
    // dynamic LDS in records of 528 floats (8 heads x 64 channels, then 8 m's, then 8 l's):
    // one record per wave (n_waves > 1), or one for the group's partial (one-wave split-K)
    extern __shared__ float lds[];
    float (*sm_acc)[8][64] = reinterpret_cast<float (*)[8][64]>(lds);
    float (*sm_m)[8] = reinterpret_cast<float (*)[8]>(lds + (blockDim.x >> 6) * 512);
    float (*sm_l)[8] = reinterpret_cast<float (*)[8]>(lds + (blockDim.x >> 6) * 520);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_waves = blockDim.x >> 6;
    const bool direct = n_waves == 1;
    const bool final_pass = prm.split_tokens == 0;
    // group-major block order, LAST chunk group first: in a ragged batch the high groups exist only
    // for the longest sequences, and dispatching them first leaves the dense low groups -- work for
    // every CU -- for the end of the kernel instead of a thin tail of a few long sequences
    const int bg = blockIdx.x % (prm.B * prm.Hkv);
    const int cgrp = (int)(gridDim.x / (prm.B * prm.Hkv)) - 1 - (int)(blockIdx.x / (prm.B * prm.Hkv));
    const int b = bg / prm.Hkv, g = bg % prm.Hkv;
    // heads of this virtual KV head: a group above 8 is cut into parts of prm.G heads, the last part may be
    // smaller (or empty: then there is nothing to do)
    const int part = g & ((1 << prm.head_shift) - 1);
    const int G = min(prm.G, prm.G_full - part * prm.G);
    const int q_first = (g >> prm.head_shift) * prm.G_full + part * prm.G;   // first query head of the part
    if (G <= 0) return;
    const int n = lane & 15, kb = lane >> 4;
    const int head = n & 7;
    const int qh = q_first + head;                       // only meaningful when head < G

    // One-wave workgroups of full-attention layers know their first step without the sequence
    // length, so their first block-table read is issued beside the read of the length instead
    // of after it (entries past the context are replaced below, before any use).
    const int32_t *bt = prm.block_table + (int64_t)b * prm.max_pages;
    const bool early_ids = direct && prm.window == 0;
    const int early_s0 = final_pass ? 0 : (cgrp * prm.chunks_per_group * prm.split_tokens) >> 6;
    int early0 = 0, early1 = 0;
    if (early_ids) {
        early0 = bt[min(early_s0 * NPS + lane, prm.max_pages - 1)];
        early1 = bt[min(early_s0 * NPS + 64 + lane, prm.max_pages - 1)];
    }

    const int L = bounded_len(prm.seq_lens[b], prm.max_len);
    const int lo = (prm.window > 0 && L > prm.window) ? L - prm.window : 0;
    const int a0 = lo & ~63;
    const int c_first = cgrp * prm.chunks_per_group;   // first chunk of this workgroup
    const int c_last = final_pass ? 1 : min(c_first + prm.chunks_per_group, prm.n_splits);
    int j0 = lo, j1 = L;
    if (!final_pass) {
        j0 = max(lo, a0 + c_first * prm.split_tokens);
        j1 = (int)min((int64_t)L, (int64_t)a0 + (int64_t)c_last * prm.split_tokens);
    }
    const bool empty = j0 >= j1;                       // uniform over the workgroup

    WaveState st;
    auto reset_state = [&]() {
        st.m = -INFINITY;
        st.l = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < 4; ++c) st.o[c] = f32x4{0.f, 0.f, 0.f, 0.f};
    };
    reset_state();

    // direct mode: put the state into LDS as the group's partial (split-K; it goes to HBM row-wise,
    // 16 lanes per 256-byte row, when the wave is done), or write it as the final row (single pass)
    auto emit_direct = [&]() {
        constexpr int slot = 0;
        const float l = add_ror8(st.l[0]);           // both P halves, all 64 positions of every step
        float scale = 1.0f;
        if (final_pass) {
            const float sink2 = (prm.sinks != nullptr && head < G) ? prm.sinks[qh] * kLog2e : -INFINITY;
            const float M = fmaxf(st.m, sink2);
            const float f = (st.m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(st.m - M);
            const float den = l * f + ((sink2 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(sink2 - M));
            scale = (den > 0.f) ? prm.v_scale * f / den : 0.f;
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            f32x4 x;
#pragma unroll
            for (int r = 0; r < 4; ++r) x[r] = add_ror8(st.o[c][r]) * scale;
            if (n < 8 && head < G) {
                if (final_pass) {
                    const int64_t at = ((int64_t)b * prm.Hq + qh) * 64 + 16 * c + 4 * kb;
                    if (prm.out_dtype == 0) {
                        *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(prm.out) + at) = x;
                    } else {
#pragma unroll
                        for (int r = 0; r < 4; ++r) store_out(prm.out, 1, at + r, x[r]);
                    }
                } else {
                    *reinterpret_cast<f32x4 *>(&lds[slot * 528 + n * 64 + 16 * c + 4 * kb]) = x;
                }
            }
        }
        if (!final_pass && lane < 8) {
            lds[slot * 528 + 512 + lane] = st.m * kLn2;
            lds[slot * 528 + 520 + lane] = l;
        }
        reset_state();
    };

    if (!empty) {
        const int s_begin = j0 >> 6, s_end = (j1 + 63) >> 6;
        const int n_steps = s_end - s_begin;
        const int s0 = s_begin + (int)(((int64_t)n_steps * wave) / n_waves);
        const int s1 = s_begin + (int)(((int64_t)n_steps * (wave + 1)) / n_waves);
        if (s0 < s1)
            run_steps<P, EB>(prm, st, bt, b, g, G, q_first, lane, L, lo, j0, j1, s0, s1, early_ids, early0, early1);
    }

    if (direct) {
        if (final_pass) {
            emit_direct();
            return;
        }
        if (empty) return;                             // no chunk of the group holds a position: nothing is written
        emit_direct();
        // the group's partial goes out through LDS: 16 lanes cover one 256-byte row, a wave-wide
        // store covers 4 rows.  The stores are non-temporal: a partial is read once, by another
        // kernel, and written through it does not wait in L2 for the write-back at the end of the
        // kernel.  Chunks of the group that lie beyond the context are not written at all: the merge
        // kernel bounds its reads by the sequence length.
        __syncthreads();                               // lanes read what other lanes put there
        const int n_rows = G;
        const int quad = lane & 15;
        for (int r0 = 0; r0 < n_rows; r0 += 16) {
            f32x4 x[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int r = min(r0 + 4 * u + (lane >> 4), n_rows - 1);
                const int cl = r / G, h = r - cl * G;
                x[u] = *reinterpret_cast<const f32x4 *>(&lds[cl * 528 + h * 64 + 4 * quad]);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int r = r0 + 4 * u + (lane >> 4);
                if (r < n_rows) {
                    const int cl = r / G, h = r - cl * G;
                    const int64_t row = ((int64_t)b * prm.Hq + q_first + h) * prm.n_splits + c_first + cl;
                    __builtin_nontemporal_store(x[u], reinterpret_cast<f32x4 *>(prm.ws_acc + row * 64 + 4 * quad));
                }
            }
        }
        // (m, l) pairs: one lane per (chunk, head)
        for (int r = lane; r < n_rows; r += 64) {
            const int cl = r / G, h = r - cl * G;
            const int64_t row = ((int64_t)b * prm.Hq + q_first + h) * prm.n_splits + c_first + cl;
            float2 ml;
            ml.x = lds[cl * 528 + 512 + h];
            ml.y = lds[cl * 528 + 520 + h];
            __builtin_nontemporal_store(ml.x, prm.ws_ml + row * 2);
            __builtin_nontemporal_store(ml.y, prm.ws_ml + row * 2 + 1);
        }
        // the group's other chunks that hold positions: empty rows
        const int c_end = min(c_last, (j1 - 1 - a0) / prm.split_tokens + 1);
        const int n_rest = (c_end - c_first - 1) * G;
        for (int r = lane; r < n_rest; r += 64) {
            const int cl = 1 + r / G, h = r % G;
            const int64_t row = ((int64_t)b * prm.Hq + q_first + h) * prm.n_splits + c_first + cl;
            __builtin_nontemporal_store(-INFINITY, prm.ws_ml + row * 2);
            __builtin_nontemporal_store(0.0f, prm.ws_ml + row * 2 + 1);
        }
        return;
    }

    // n_waves > 1: per-wave result -> LDS (the two P halves added), then merge and write the final
    // row or the sink-free partial; a split-K chunk beyond the context is not written at all
    if (empty && !final_pass) return;
    const float l = add_ror8(st.l[0]);
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float x = add_ror8(st.o[c][r]);
            if (n < 8) sm_acc[wave][n][16 * c + 4 * kb + r] = x;
        }
    if (lane < 8) {
        sm_m[wave][lane] = st.m;
        sm_l[wave][lane] = l;
    }
    __syncthreads();

    for (int idx = threadIdx.x; idx < G * 64; idx += blockDim.x) {
        const int h = idx >> 6, c = idx & 63;
        const int qhead = q_first + h;
        float M = -INFINITY;
        for (int w = 0; w < n_waves; ++w) M = fmaxf(M, sm_m[w][h]);
        float sink2 = -INFINITY;
        if (final_pass && prm.sinks != nullptr) sink2 = prm.sinks[qhead] * kLog2e;
        M = fmaxf(M, sink2);
        float num = 0.f, den = 0.f;
        if (M != -INFINITY) {
            den = (sink2 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(sink2 - M);
            for (int w = 0; w < n_waves; ++w) {
                const float mw = sm_m[w][h];
                if (mw == -INFINITY) continue;
                const float f = __builtin_amdgcn_exp2f(mw - M);
                num = __builtin_fmaf(sm_acc[w][h][c], f, num);
                den = __builtin_fmaf(sm_l[w][h], f, den);
            }
        }
        if (final_pass) {
            const float r = (den > 0.f) ? prm.v_scale * num / den : 0.f;
            store_out(prm.out, prm.out_dtype, ((int64_t)b * prm.Hq + qhead) * 64 + c, r);
        } else {
            const int64_t row = ((int64_t)b * prm.Hq + qhead) * prm.n_splits + c_first;
            prm.ws_acc[row * 64 + c] = num;
            if (c == 0) {
                prm.ws_ml[row * 2] = M * kLn2;
                prm.ws_ml[row * 2 + 1] = den;
            }
        }
    }
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x = fmaxf(x, __shfl_xor(x, d));
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d);
    return x;
}

// Merge kernel: one workgroup of W waves per (sequence, query head).  The chunks are taken 64 at a
// time (wave w takes batches w, w + W, ...): lane i fetches (m_i, l_i) of chunk i and computes its
// weight exp(m_i - M); then lane = channel and the 64 accumulator rows are streamed, all 64 loads
// of a lane in flight together, each row scaled by its chunk's weight read out of the weight
// register (uniform lane index).  A wave's first batch is fetched before the sequence length is
// known; rows of chunks beyond the sequence (which the first pass does not write) are inside the
// workspace, so the read is safe, and they are discarded.  With W > 1 (more than 64 chunks: each
// batch is a dependent round trip to memory, so they are spread over four or eight waves) the waves' running
// (M, numerator, denominator) meet in LDS and wave 0, which also carries the sink, finishes.
// NB = chunks per batch (64, or 16 for rows of at most 16 chunks so that a short row does not issue 64 loads).
// LAZY: the accumulator rows are fetched after the (m, l) pairs, only those that hold a partial.
// D: head dimension; with 128 a second grid row of workgroups merges channels 64..127 the same way.
template <int W, int NB, bool LAZY = false, int D = 64>
__global__ __launch_bounds__(64 * W) void splitk_reduce_kernel(const pz::ReduceParams prm) {
    const int row = blockIdx.x;                        // b * Hq + h
    const int b = row / prm.Hq, h = row % prm.Hq;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int S = prm.n_splits;
    const float *acc = prm.ws_acc + (int64_t)row * S * D + (D > 64 ? 64 * (int)blockIdx.y : 0);
    const float2 *ml = reinterpret_cast<const float2 *>(prm.ws_ml) + (int64_t)row * S;
    const float sink = (prm.sinks != nullptr && wave == 0) ? prm.sinks[h] : -INFINITY;
    float M = sink;                                    // running reference maximum
    float num = 0.f;
    float den = (sink == -INFINITY) ? 0.f : 1.0f;      // exp(sink - M) with M == sink
    int n = S;
    bool first = true;
    for (int base = NB * wave; base < n; base += NB * W) {
        const int cnt = min(NB, S - base);             // rows that exist
        float2 v = {-INFINITY, 0.f};
        if (lane < cnt) v = ml[base + lane];
        const float *a = acc + (int64_t)base * D + lane;
        float x[NB];
        if constexpr (!LAZY) {
#pragma unroll
            for (int u = 0; u < NB; ++u) x[u] = __builtin_nontemporal_load(a + (int64_t)min(u, cnt - 1) * D);
        }
        if (first && prm.seq_lens != nullptr) {        // chunks past this bound were never written
            const int L = bounded_len(prm.seq_lens[b], 1 << 30);   // keeps the sums below in 32 bits
            const int lo = (prm.window > 0 && L > prm.window) ? L - prm.window : 0;
            const int span = L - (lo & ~63);
            n = min(S, (span + prm.split_tokens - 1) / prm.split_tokens);
        }
        first = false;
        if (base + lane >= n) v = float2{-INFINITY, 0.f};
        const float M_new = fmaxf(M, wave_max(v.x));
        if (M_new == -INFINITY) continue;              // only empty partials so far, no sink
        const float keep = (M == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((M - M_new) * kLog2e);
        const float w = (v.x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((v.x - M_new) * kLog2e);
        num *= keep;
        den = den * keep + wave_sum(v.y * w);
        M = M_new;
        if constexpr (LAZY) {
            // only the rows that hold a partial are fetched, eight at a time (all eight loads in flight)
            uint64_t live = __ballot(w != 0.f && base + lane < n);
            while (live != 0) {
                int idx[8];
                float xv[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    idx[e] = live != 0 ? __builtin_ctzll(live) : -1;
                    if (live != 0) live &= live - 1;
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) xv[e] = __builtin_nontemporal_load(a + (int64_t)max(idx[e], 0) * D);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float we = __shfl(w, max(idx[e], 0));
                    num = __builtin_fmaf(idx[e] >= 0 ? xv[e] : 0.f, idx[e] >= 0 ? we : 0.f, num);
                }
            }
            continue;
        }
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const float wu = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w), u));
            // rows past the sequence's chunks may hold anything (the first batch is fetched before
            // the bound is known), and so may the acc of an empty row (its chunk was merged into an
            // earlier row and only its (m, l) were written): both are dropped by a select, not by a
            // zero weight
            num = __builtin_fmaf((base + u < n && wu != 0.f) ? x[u] : 0.f, wu, num);
        }
    }
    if constexpr (W > 1) {
        __shared__ float part[W][66];                  // numerator[64], M, denominator of every wave
        part[wave][lane] = num;
        if (lane == 0) {
            part[wave][64] = M;
            part[wave][65] = den;
        }
        __syncthreads();
        if (wave != 0) return;
        float M_all = M;
#pragma unroll
        for (int w = 1; w < W; ++w) M_all = fmaxf(M_all, part[w][64]);
        if (M_all != -INFINITY) {
            const float f0 = (M == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((M - M_all) * kLog2e);
            num *= f0;
            den *= f0;
#pragma unroll
            for (int w = 1; w < W; ++w) {
                const float Mw = part[w][64];
                const float f = (Mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((Mw - M_all) * kLog2e);
                num = __builtin_fmaf(part[w][lane], f, num);
                den = __builtin_fmaf(part[w][65], f, den);
            }
        }
    }
    const float r = (den > 0.f) ? prm.v_scale * num / den : 0.f;
    store_out(prm.out, prm.out_dtype, (int64_t)row * D + (D > 64 ? 64 * (int)blockIdx.y : 0) + lane, r);
}

}  // namespace

namespace pz {

hipError_t launch_decode_attn(const AttnParams &prm, int page_size, int elem_bytes, int n_waves,
                              hipStream_t stream) {
    const int n_chunks = prm.split_tokens > 0 ? prm.n_splits : 1;
    const int n_groups = (n_chunks + prm.chunks_per_group - 1) / prm.chunks_per_group;
    const dim3 grid((unsigned)(prm.B * prm.Hkv * n_groups)), block(64 * n_waves);
    const size_t records = n_waves > 1 ? n_waves : (prm.split_tokens > 0 ? 1 : 0);
    const size_t lds_bytes = records * (8 * 64 + 16) * sizeof(float);
#define PZ_LAUNCH(P, EB) return launch(decode_attn_kernel<P, EB>, grid, block, lds_bytes, stream, prm)
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

hipError_t launch_splitk_reduce(const ReduceParams &prm, hipStream_t stream) {
    // one wave per 64 chunks, at most eight; short rows in one batch of 16
    if (prm.head_dim == 128) {
        const dim3 grid((unsigned)(prm.B * prm.Hq), 2);
        if (prm.n_splits <= 16) return launch(splitk_reduce_kernel<1, 16, false, 128>, grid, dim3(64), 0, stream, prm);
        if (prm.n_splits <= 64) return launch(splitk_reduce_kernel<1, 64, false, 128>, grid, dim3(64), 0, stream, prm);
        if (prm.n_splits <= 256) return launch(splitk_reduce_kernel<4, 64, false, 128>, grid, dim3(256), 0, stream, prm);
        return launch(splitk_reduce_kernel<8, 64, false, 128>, grid, dim3(512), 0, stream, prm);
    }
    const dim3 grid((unsigned)(prm.B * prm.Hq));
    if (prm.n_splits <= 16) return launch(splitk_reduce_kernel<1, 16>, grid, dim3(64), 0, stream, prm);
    // A job this large was walked by one-wave workgroups that each merged a run of chunks in registers (at
    // least 2048 (sequence, KV head, chunk) items whatever the group size), so most rows are empty markers:
    // the accumulator rows are then asked for once the (m, l) pairs show which ones hold a partial -- a
    // dependent round trip instead of 64 row loads per lane of which 56 are dropped (batch 16 x 64K:
    // 171.9 -> 170.0 us per step, batch 32 x 64K 328.8 -> 324.2).  Smaller jobs have a partial in every row
    // and fetch everything at once.
    const bool lazy = (int64_t)prm.B * prm.Hq * prm.n_splits >= 16384;
#define PZ_REDUCE(W) (lazy ? launch(splitk_reduce_kernel<W, 64, true>, grid, dim3(64 * W), 0, stream, prm) \
                           : launch(splitk_reduce_kernel<W, 64, false>, grid, dim3(64 * W), 0, stream, prm))
    // Never two waves per workgroup: a grid of two-wave workgroups leaves the chip in a state in which the
    // one-wave workgroups of the attention launch that follows are placed unevenly over the SIMDs (that launch
    // then took 11 to 13 us longer: ragged batch 32 at 1024-token chunks 325 -> 312 us per attention + merge,
    // batch 8 x 128K 174 -> 168); one, four and eight waves per workgroup do not.  65 to 128 chunks therefore
    // run on four waves, two of them idle.
    if (prm.n_splits <= 64) return PZ_REDUCE(1);
    if (prm.n_splits <= 256) return PZ_REDUCE(4);
    return PZ_REDUCE(8);
#undef PZ_REDUCE
}

}  // namespace pz
