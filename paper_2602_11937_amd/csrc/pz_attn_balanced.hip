// Split-K decode attention with a balanced partition of the chunks for gfx950 (MI355X).
//
// Same operation and same per-step arithmetic as decode_attn_kernel (pz_attn.hip): single-token GQA
// attention over the paged FP8 / bf16 cache, sliding window ("most recent W tokens", paper Section 2,
// "Window attention for long-context inference"), sink-free partials (acc, m, l) per chunk of
// split_tokens positions.  What differs is who does which chunk.  A launch grid can only be sized
// from the longest sequence, so with one workgroup per (sequence, chunk group) a ragged batch
// leaves many workgroups empty, the rest uneven, and the kernel ends in a long thin tail.  Here
// every workgroup (one wave64) first reads all sequence lengths, counts the chunks that exist,
//     n_b = min(n_splits, ceil((L_b - a_b) / split_tokens)),   tot = sum_b n_b,
// and takes an equal share of the list (b, chunk) in sequence order for its KV head: with
// k = ceil(tot / workgroups_per_head) chunks in the largest share, n_act = ceil(tot / k) workgroups
// are active; the first tot mod n_act shares hold k chunks and the others k - 1, so the shares
// that differ have LESS work and nothing is left over at the end (balanced_plan, pz_internal.h).
// A share may span several sequences; each run of chunks inside one sequence is streamed with
// the register pipeline of pz_attn.hip as ONE online softmax, and leaves one partial: it goes to
// the workspace row of the run's first chunk, and the rows of the run's other chunks are marked
// empty (m = -inf, l = 0), which the merge kernel skips.  Merging a run in registers is the same
// arithmetic as the merge kernel's, done earlier: on batch 16 x 64K (8 chunks per run) it saves
// writing and re-reading 7 of 8 partials, 175.1 -> 172.5 us per step.  The partition is a pure
// function of the lengths: no queue, no atomics, nothing to wait for.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pz_attn_common.h"
#include "pz_attn_steps.h"
#include "pz_internal.h"
#include "pz_quant.h"

namespace {

// Inclusive prefix sum over the 64 lanes with DPP moves only (no LDS traffic): four shifted adds
// inside every row of 16 lanes, then lane 15 of rows 0 and 2 is added to rows 1 and 3, then
// lane 31 to rows 2 and 3.  Lane 63 ends up with the total.
__device__ __forceinline__ int wave_inclusive_scan_int(int x) {
    x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, true);     // row_shr:1
    x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, true);     // row_shr:2
    x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, true);     // row_shr:4
    x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, true);     // row_shr:8
    x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, false);    // row_bcast:15 into rows 1 and 3
    x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, false);    // row_bcast:31 into rows 2 and 3
    return x;
}

// The stated budget is three waves per SIMD (170 registers); the kernel takes 133 for FP8 caches with
// 64-token pages.  Asking for four waves (128 registers) makes the compiler schedule for register
// pressure and spill in the run set-up, which cost 10 %; the shares are planned for one wave per
// SIMD anyway.
template <int P, int EB>
__global__ __launch_bounds__(64, 3) void decode_attn_balanced_kernel(const pz::AttnParams prm) {
    constexpr int NPS = 64 / P;                        // pages per step
    __shared__ float lds[528];                         // a run's partial on its way out: 8 x 64 acc, 8 m, 8 l

    const int lane = threadIdx.x;
    const int n = lane & 15, kb = lane >> 4;
    const int head = n & 7;
    // Workgroup t works on share t / Hkv of KV head (t + t / Hkv) % Hkv.  The active shares are the lowest
    // ones, so the workgroups that stream are the first of the grid and are placed like a launch of
    // just that many (the idle rest is dispatched after them and leaves at once); the rotation makes
    // every XCD, which receives every eighth workgroup, stream all KV heads.
    const int bph = gridDim.x / prm.Hkv;               // workgroups per KV head
    const int i_blk = blockIdx.x / prm.Hkv;
    const int g = (blockIdx.x + i_blk) % prm.Hkv;
    // heads of this virtual KV head: a group above 8 is cut into parts of prm.G heads, the last part may be
    // smaller (or empty: then there is nothing to do)
    const int part = g & ((1 << prm.head_shift) - 1);
    const int G = min(prm.G, prm.G_full - part * prm.G);
    const int q_first = (g >> prm.head_shift) * prm.G_full + part * prm.G;   // first query head of the part
    if (G <= 0) return;
    const int split = prm.split_tokens;
    const int steps_per_chunk = split >> 6;

    auto chunks_of = [&](int L) -> int {
        if (L <= 0) return 0;
        const int lo = (prm.window > 0 && L > prm.window) ? L - prm.window : 0;
        const int span = L - (lo & ~63);
        return min(prm.n_splits, (span + split - 1) / split);
    };
    // the share of this workgroup out of `tot` chunks: [begin, end) of the list, or nothing.  The host
    // keeps batch * n_kv_heads * n_splits below 2^31, so 32-bit arithmetic is enough.
    auto pick = [&](unsigned n_act, unsigned q, unsigned r, unsigned &begin, unsigned &end) -> bool {
        const unsigned i = (unsigned)i_blk;
        if (i >= n_act) return false;
        begin = i * q + min(i, r);                     // the first r shares hold q + 1 chunks
        end = begin + q + (i < r ? 1u : 0u);
        return true;
    };
    auto share = [&](unsigned tot, unsigned &begin, unsigned &end) -> bool {
        if (tot == 0) return false;
        unsigned n_act, q, r;
        pz::balanced_plan(tot, (unsigned)prm.Hkv, (unsigned)bph, &n_act, &q, &r);
        return pick(n_act, q, r, begin, end);
    };

    // Before the lengths are known: if every sequence had the longest length this workgroup would
    // start at (spec_b, spec_c); the block-table entries of that place are fetched beside the
    // lengths and used when the guess holds (it always does for a uniform batch).
    const unsigned tot_full = (unsigned)prm.B * (unsigned)prm.n_splits;
    unsigned spec_begin = 0, spec_end = 0;
    const bool spec_active = pick(prm.full_n_act, prm.full_q, prm.full_r, spec_begin, spec_end);
    int spec_b = -1, spec_c = 0, early0 = 0, early1 = 0;
    if (spec_active && prm.window == 0) {
        spec_b = (int)(spec_begin / (unsigned)prm.n_splits);
        spec_c = (int)(spec_begin - (unsigned)spec_b * (unsigned)prm.n_splits);
        const int32_t *row = prm.block_table + (int64_t)spec_b * prm.max_pages;
        const int p0 = spec_c * steps_per_chunk * NPS;
        early0 = row[min(p0 + lane, prm.max_pages - 1)];
        early1 = row[min(p0 + 64 + lane, prm.max_pages - 1)];
    }

    // chunk count of the batch and, for the first 64 sequences, the lengths and prefix sums
    unsigned tot = 0;
    int len0 = 0, nn0 = 0, incl0 = 0;
    bool found = false;                                // (b, c, L_first) already known
    int b = 0, c = 0, L_first = 0;
    {
        // all lengths equal and full: the guess above is the answer, no sums needed
        const int L0 = bounded_len(prm.seq_lens[0], prm.max_len);
        bool uniform = spec_b >= 0 && chunks_of(L0) == prm.n_splits;
        for (int base = 0; base < prm.B && uniform; base += 64) {
            const int L = (base + lane < prm.B) ? bounded_len(prm.seq_lens[base + lane], prm.max_len) : L0;
            uniform = __ballot(L != L0) == 0;
        }
        if (uniform) {
            if (!spec_active) return;
            found = true;
            tot = tot_full;
            b = spec_b;
            c = spec_c;
            L_first = L0;
        }
    }
    for (int base = 0; base < prm.B && !found; base += 64) {
        const int L = (base + lane < prm.B) ? bounded_len(prm.seq_lens[base + lane], prm.max_len) : 0;
        const int nn = chunks_of(L);
        const int incl = wave_inclusive_scan_int(nn);
        if (base == 0) {
            len0 = L;
            nn0 = nn;
            incl0 = incl;
        }
        tot += __builtin_amdgcn_readlane(incl, 63);     // uniform: stays scalar
    }
    unsigned c_begin = spec_begin, c_end = spec_end;
    if (tot != tot_full) {
        if (!share(tot, c_begin, c_end)) return;
    } else if (!spec_active) {
        return;
    }

    // the sequence that holds list entry c_begin, the chunk inside it, and the sequence's length
    if (!found) {
        unsigned run = 0;
        for (int base = 0; base < prm.B; base += 64) {
            int len = len0, nn = nn0, incl = incl0;
            if (base > 0) {
                len = (base + lane < prm.B) ? bounded_len(prm.seq_lens[base + lane], prm.max_len) : 0;
                nn = chunks_of(len);
                incl = wave_inclusive_scan_int(nn);
            }
            const uint64_t past = __ballot(run + (unsigned)incl > c_begin);
            if (past != 0) {
                const int l0 = __builtin_ctzll(past);
                b = base + l0;
                c = (int)(c_begin - (run + __builtin_amdgcn_readlane(incl, l0) - __builtin_amdgcn_readlane(nn, l0)));
                L_first = __builtin_amdgcn_readlane(len, l0);
                break;
            }
            run += __builtin_amdgcn_readlane(incl, 63);
        }
        b = min(b, prm.B - 1);                         // c_begin < tot puts (b, c) inside the batch anyway
        c = max(c, 0);
    }

    WaveState st;
    auto reset_state = [&]() {
        st.m = -INFINITY;
        st.l = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) st.o[cc] = f32x4{0.f, 0.f, 0.f, 0.f};
    };
    reset_state();

    // put the state into LDS as the run's partial and reset it
    auto park = [&]() {
        constexpr int slot = 0;
        const float l = add_ror8(st.l[0]);             // both P halves, all 64 positions of every step
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
            f32x4 x;
#pragma unroll
            for (int r = 0; r < 4; ++r) x[r] = add_ror8(st.o[cc][r]);
            if (n < 8 && head < G) *reinterpret_cast<f32x4 *>(&lds[slot * 528 + n * 64 + 16 * cc + 4 * kb]) = x;
        }
        if (lane < 8) {
            lds[slot * 528 + 512 + lane] = st.m * kLn2;
            lds[slot * 528 + 520 + lane] = l;
        }
        reset_state();
    };
    // write the parked partial of the run [chunk0, chunk_end) of sequence bb to the rows of chunk0 and
    // mark the rows of the other chunks empty: 16 lanes cover one 256-byte row, a wave-wide store covers
    // 4 rows.  Non-temporal: read once, by the merge kernel.
    auto write_out = [&](int bb, int chunk0, int chunk_end) {
        __syncthreads();                               // lanes read what other lanes parked
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
                    const int64_t row = ((int64_t)bb * prm.Hq + q_first + h) * prm.n_splits + chunk0 + cl;
                    __builtin_nontemporal_store(x[u], reinterpret_cast<f32x4 *>(prm.ws_acc + row * 64 + 4 * quad));
                }
            }
        }
        for (int r = lane; r < n_rows; r += 64) {      // (m, l) pairs: one lane per (chunk, head)
            const int cl = r / G, h = r - cl * G;
            const int64_t row = ((int64_t)bb * prm.Hq + q_first + h) * prm.n_splits + chunk0 + cl;
            __builtin_nontemporal_store(lds[cl * 528 + 512 + h], prm.ws_ml + row * 2);
            __builtin_nontemporal_store(lds[cl * 528 + 520 + h], prm.ws_ml + row * 2 + 1);
        }
        const int n_rest = (chunk_end - chunk0 - 1) * G;
        for (int r = lane; r < n_rest; r += 64) {
            const int cl = 1 + r / G, h = r % G;
            const int64_t row = ((int64_t)bb * prm.Hq + q_first + h) * prm.n_splits + chunk0 + cl;
            __builtin_nontemporal_store(-INFINITY, prm.ws_ml + row * 2);
            __builtin_nontemporal_store(0.0f, prm.ws_ml + row * 2 + 1);
        }
        __syncthreads();                               // the record is free again
    };

    bool first_run = true;
    int remaining = (int)(c_end - c_begin);
    int L = L_first;                                   // length of sequence b
    while (remaining > 0) {
        const int nb = chunks_of(L);
        if (c >= nb) {                                 // sequence used up (or without chunks): next one
            if (++b >= prm.B) break;                   // cannot happen while chunks remain; keeps the loop finite
            L = bounded_len(prm.seq_lens[b], prm.max_len);
            c = 0;
            continue;
        }
        const int c_first = c;
        const int c_last = c + min(nb - c, remaining);
        remaining -= c_last - c_first;
        c = c_last;

        // ---- one run: chunks [c_first, c_last) of sequence b
        const int32_t *bt = prm.block_table + (int64_t)b * prm.max_pages;
        const int lo = (prm.window > 0 && L > prm.window) ? L - prm.window : 0;
        const int a0 = lo & ~63;
        const int j0 = max(lo, a0 + c_first * split);
        const int j1 = (int)min((int64_t)L, (int64_t)a0 + (int64_t)c_last * split);
        const int s0 = j0 >> 6, s1 = (j1 + 63) >> 6;   // s0 < s1: every chunk of the list holds a position
        const bool use_early = first_run && b == spec_b && c_first == spec_c;   // then s0 == spec_c * steps_per_chunk
        first_run = false;
        run_steps<P, EB>(prm, st, bt, b, g, G, q_first, lane, L, lo, j0, j1, s0, s1, use_early, early0, early1);
        park();
        write_out(b, c_first, c_last);
    }
}

}  // namespace

namespace pz {

// Workgroups of decode_attn_balanced_kernel<P, EB> (one wave each) that fit the device at once: the
// partition never plans more shares per launch than this.  Worked out once per kernel variant
// (function-local static: initialised once, also with several host threads).
template <int P, int EB>
static int query_slots() {
    int per_cu = 0, dev = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_attn_balanced_kernel<P, EB>, 64, 0) !=
            hipSuccess || per_cu <= 0)
        per_cu = 8;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        cus = 256;
    return per_cu * cus;
}

template <int P, int EB>
static int slots_of() {
    static const int slots = query_slots<P, EB>();
    return slots;
}

static int balanced_slots(int page_size, int elem_bytes) {
    if (elem_bytes == 1) return page_size == 64 ? slots_of<64, 1>() : (page_size == 32 ? slots_of<32, 1>() : slots_of<16, 1>());
    return page_size == 64 ? slots_of<64, 2>() : (page_size == 32 ? slots_of<32, 2>() : slots_of<16, 2>());
}

hipError_t launch_decode_attn_balanced(const AttnParams &prm_in, int page_size, int elem_bytes, hipStream_t stream) {
    // workgroups per KV head: twice as many as the kernel activates when every sequence has the longest
    // length (shorter sequences mean fewer chunks, for which the plan may want smaller shares and hence up
    // to twice the workgroups), never more than there are chunks or than fit the device at once
    AttnParams prm = prm_in;
    const unsigned cap_chunks = (unsigned)prm.B * (unsigned)prm.n_splits;
    unsigned bph = (unsigned)(balanced_slots(page_size, elem_bytes) / prm.Hkv);
    if (bph < 1) bph = 1;
    balanced_plan(cap_chunks, (unsigned)prm.Hkv, bph, &prm.full_n_act, &prm.full_q, &prm.full_r);
    {
        unsigned room = prm.full_n_act * 2u;
        if (room > cap_chunks) room = cap_chunks;
        if (room > bph) room = bph;
        bph = room < prm.full_n_act ? prm.full_n_act : room;
    }
    const dim3 grid((unsigned)(bph * prm.Hkv)), block(64);
#define PZ_LAUNCH(PP, EE) return launch(decode_attn_balanced_kernel<PP, EE>, grid, block, 0, stream, prm)
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
