// Internal launch interface between the C-ABI layer (pz_api.hip) and the kernels.
#ifndef PZ_INTERNAL_H
#define PZ_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <tuple>
#include <utility>

namespace pz {

// Enqueue `kernel` and return the status of THIS launch.  hipLaunchKernel hands back its own result, so an
// error that earlier, unrelated work left behind on the calling thread is neither reported as this call's
// nor cleared by it (a launch followed by hipGetLastError would do both).
template <typename... KArgs, size_t... I>
inline hipError_t launch_impl(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream,
                              std::tuple<KArgs...> &vals, std::index_sequence<I...>) {
    void *ptrs[] = {static_cast<void *>(&std::get<I>(vals))...};
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, lds_bytes, stream);
}
template <typename... KArgs, typename... Args>
inline hipError_t launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream,
                         Args &&...args) {
    static_assert(sizeof...(KArgs) == sizeof...(Args), "one argument per kernel parameter");
    std::tuple<KArgs...> vals{static_cast<KArgs>(args)...};
    return launch_impl(kernel, grid, block, lds_bytes, stream, vals, std::index_sequence_for<KArgs...>{});
}

// Launch-shape overrides set through pz_debug_set_launch_override (tests and measurements); the value of
// an override that is not set is negative.  Indexed by pz_launch_override.
int launch_override(int which);

struct AttnParams {
    uint8_t *k;                  // K cache  [page][Hkv][P][d]   (written only by the fused append); d = 64 or 128
    uint8_t *v;                  // V cache  [page][Hkv][d][P]
    const uint16_t *q;           // bf16 [B][Hq][d]
    const int32_t *block_table;  // [B][max_pages]
    const int32_t *seq_lens;     // [B]
    const float *sinks;          // [Hq] or nullptr
    float *ws_acc;               // split-K partials [B][Hq][S][64]
    float *ws_ml;                // [B][Hq][S][2]
    void *out;                   // [B][Hq][64]
    // fused append (both nullptr: none): the newest token's K/V rows, bf16 [B][cache_heads][64].  The wave
    // that attends position L_b - 1 takes them from here, quantised in registers, and writes them into the
    // cache after its last step
    const uint16_t *k_new;
    const uint16_t *v_new;
    float k_scale;               // for the fused append only (the logits use sc)
    int32_t max_pages, B, Hq, Hkv, G;   // Hkv, G: "virtual" KV heads of at most 8 query heads each
    int32_t cache_heads, head_shift;    // KV heads of the cache; virtual head g reads cache head g >> head_shift
    int32_t G_full;                     // query heads per cache KV head (G = heads per virtual head, the part size)
    int32_t window, split_tokens, n_splits, out_dtype;
    int32_t chunks_per_group;    // consecutive split-K chunks walked by one workgroup (1 unless it is one wave)
    // balanced kernel: the partition of a batch whose sequences all have n_splits chunks, worked out on
    // the host (n_act shares; the first r hold q + 1 chunks, the others q)
    uint32_t full_n_act, full_q, full_r;
    // what device-side inputs are held to, so that no access leaves the cache or a block-table row whatever
    // they contain: lengths are cut to max_len = max_pages * page_size, page ids to [0, num_pages)
    int32_t num_pages, max_len;
    float sc;                    // sm_scale * k_scale * log2(e)
    float v_scale;
};

hipError_t launch_decode_attn_balanced(const AttnParams &prm, int page_size, int elem_bytes, hipStream_t stream);
// head dimension 128 (pz_attn_d128.hip): one-wave workgroups per (sequence, KV head, chunk group)
hipError_t launch_decode_attn_d128(const AttnParams &prm, int page_size, int elem_bytes, hipStream_t stream);

// Balanced partition of `tot` chunks of one KV head over at most `bph` workgroups: n_act shares, the
// first r of q + 1 chunks, the others of q.  The share size aimed at is the smallest that leaves at
// most 1024 waves over all heads -- one per SIMD, four per CU; measured best on this chip, ahead of
// twice or four times as many shorter shares and far ahead of counts that fill the CUs unevenly --
// so never more than 1024 shares in all, however many chunks there are.  With k = q + 1 (or q when
// r == 0) the largest share, n_act = ceil(tot / k), so the shares that differ are the smaller ones.
__host__ __device__ inline unsigned balanced_want(unsigned tot, unsigned n_heads) {
    const unsigned want = (tot * n_heads + 1023u) / 1024u;
    return want < 1u ? 1u : want;
}
__host__ __device__ inline void balanced_plan(unsigned tot, unsigned n_heads, unsigned bph, unsigned *n_act,
                                              unsigned *q, unsigned *r) {
    const unsigned want = balanced_want(tot, n_heads);
    unsigned cap = (tot + want - 1u) / want;
    const unsigned simds_per_head = n_heads >= 1024u ? 1u : 1024u / n_heads;
    if (cap > simds_per_head) cap = simds_per_head;    // head counts that do not divide 1024
    if (cap > bph) cap = bph;
    const unsigned k = (tot + cap - 1u) / cap;
    *n_act = (tot + k - 1u) / k;
    *q = tot / *n_act;
    *r = tot - *q * *n_act;
}

struct ReduceParams {
    const float *ws_acc;
    const float *ws_ml;
    const int32_t *seq_lens;     // or nullptr
    const float *sinks;          // or nullptr
    void *out;
    int32_t B, Hq, n_splits, window, split_tokens, out_dtype;
    int32_t head_dim;            // 64 or 128: row length of ws_acc and of out
    float v_scale;
};

struct AppendParams {
    uint8_t *k;                  // K cache
    uint8_t *v;                  // V cache
    const uint16_t *k_new;       // bf16 [T][Hkv][64]
    const uint16_t *v_new;
    const int64_t *slot_mapping; // [T]
    int64_t T;
    int64_t num_slots;           // num_pages * P: tokens whose slot is not in [0, num_slots) are skipped
    int32_t Hkv, P;
    int32_t D;                   // head dimension, 64 or 128 (the kernels then run once per 64-channel half)
    float k_scale, v_scale;
};

#ifndef PZ_PREFILL_NT
#define PZ_PREFILL_NT 3          // column tiles per wave of the prefill kernel: 2 * NT query tokens
#endif

struct PrefillParams {
    const uint8_t *k;
    const uint8_t *v;
    const uint16_t *q;           // bf16 [T][Hq][64], the new tokens of a sequence contiguous, in order
    const int32_t *q_start;      // [B + 1] offsets into T
    const int32_t *block_table;
    const int32_t *seq_lens;     // [B], counting the new tokens
    const float *sinks;
    void *out;                   // [T][Hq][64]
    int32_t max_pages, B, Hq, Hkv, G, window, out_dtype, tiles_per_seq;   // Hkv, G: virtual heads as in AttnParams
    int32_t cache_heads, head_shift, G_full;
    int32_t num_pages, max_len;  // bounds for page ids and lengths, as in AttnParams
    float sc, v_scale;
};

hipError_t launch_prefill_attn(const PrefillParams &prm, int page_size, int elem_bytes, int n_tiles,
                               hipStream_t stream);

struct RopeAppendParams {
    AppendParams ap;             // cache, k_new, v_new, slots, T, scales
    const uint16_t *q_in;        // bf16 [T][Hq][64]
    uint16_t *q_out;             // bf16 [T][Hq][64]
    const int32_t *positions;    // [T]
    const float *cos_tab;        // [n_pos][32]
    const float *sin_tab;
    int32_t Hq;
};

hipError_t launch_rope_kv_append(const RopeAppendParams &prm, int elem_bytes, hipStream_t stream);
hipError_t launch_decode_attn(const AttnParams &prm, int page_size, int elem_bytes, int n_waves,
                              hipStream_t stream);
hipError_t launch_splitk_reduce(const ReduceParams &prm, hipStream_t stream);
hipError_t launch_kv_append(const AppendParams &prm, int elem_bytes, hipStream_t stream);
hipError_t launch_kv_append_last(const AppendParams &prm, const int32_t *block_table, int max_pages,
                                 const int32_t *seq_lens, int batch, int elem_bytes, hipStream_t stream);
hipError_t launch_kv_amax(const uint16_t *k, const uint16_t *v, int64_t n, float *amax, hipStream_t stream);
hipError_t launch_kv_scales(const float *amax, int round_up_pow2, float *scales, hipStream_t stream);

}  // namespace pz
#endif
