// C-ABI layer: argument validation (host only, before anything is enqueued) and dispatch.
#include <hip/hip_runtime.h>
#include <math.h>

#include <atomic>

#include "pz.h"
#include "pz_internal.h"

namespace {

// launch-shape overrides (pz_debug_set_launch_override); negative = the library's own choice
std::atomic<int> g_override[PZ_OVERRIDE_COUNT] = {{-1}, {-1}, {-1}, {-1}, {-1}};

bool supported_page(int p) { return p == 16 || p == 32 || p == 64; }

// wide: the entry point also takes a head dimension of 128 (append, decode attention, merge); prefill and
// the rotary append are for 64-channel heads
pz_status check_cache(const pz_cache *c, bool wide = false) {
    if (c == nullptr || c->k == nullptr || c->v == nullptr) return PZ_ERR_NULL;
    if (c->num_pages <= 0 || c->page_size <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0) return PZ_ERR_SHAPE;
    if (c->dtype != PZ_KV_FP8_E4M3 && c->dtype != PZ_KV_BF16) return PZ_ERR_UNSUPPORTED;
    if (!(c->head_dim == 64 || (wide && c->head_dim == 128)) || !supported_page(c->page_size)) return PZ_ERR_UNSUPPORTED;
    return PZ_OK;
}

// positions per sequence the kernels' 32-bit position arithmetic is sized for
constexpr int64_t kMaxPositions = 1 << 30;

bool positive_finite(float x) { return x > 0.0f && isfinite(x); }

// Query heads per KV head the attention kernels take: a column tile holds 8 heads, so up to 8
// directly; a larger group runs as 2, 4 or 8 virtual KV heads that all read the same cache head,
// each with a part of ceil(group / parts) heads (the last part holds what is left, possibly
// nothing).  Returns log2 of the number of virtual heads per KV head, or -1 for groups above 64.
int group_shift(int group) {
    if (group < 1) return -1;
    for (int k = 0; k <= 3; ++k)
        if (((group + (1 << k) - 1) >> k) <= 8) return k;
    return -1;
}
bool group_supported(int group) { return group_shift(group) >= 0; }

int round_down_pow2(int x) {
    int r = 1;
    while (2 * r <= x) r *= 2;
    return r;
}

// Launch shape of decode_attn_kernel.  The chip holds 1024 SIMDs; a wave streams best when it owns a
// long run of steps (its start-up and its final store are latency it cannot hide), so:
//   - with plenty of chunks, one-wave workgroups each walk several consecutive chunks
//     (chunks_per_group) as one run: the sequence's `full_chunks` whole chunks are cut into as few
//     even groups as leave about one wave per SIMD or more (a window of 8192 positions in 1024-token
//     chunks is 8 whole chunks and a last one of at most 63 positions; measured at batch 32 / 64 /
//     128 / 256: groups of 2 / 4 / 9 / 9 chunks are fastest, 47.7 / 88.9 / 164.7 / 325.8 us).
//     Full-attention split-K goes to decode_attn_balanced_kernel instead, which deals the chunks out
//     on the device; window layers and single-pass calls stay here;
//   - with few (sequence, KV head, chunk) items, the steps of one item are dealt to several waves.
void pick_shape(int batch, int n_kv_heads, int max_steps, int n_chunks, int full_chunks, int *n_waves,
                int *chunks_per_group) {
    const long items = (long)batch * n_kv_heads * n_chunks;
    const int forced_w = pz::launch_override(PZ_OVERRIDE_ATTN_WAVES);
    const int forced_c = pz::launch_override(PZ_OVERRIDE_ATTN_CHUNKS_PER_GROUP);
    int w = 1;
    if (forced_w > 0) w = forced_w > 8 ? 8 : round_down_pow2(forced_w);
    else while (w < 8 && items * w < 2048 && max_steps >= 4 * w) w *= 2;
    int c = 1;
    if (w == 1 && n_chunks > 1) {
        if (forced_c > 0) {
            c = forced_c;
        } else {
            const long pairs = (long)batch * n_kv_heads;
            long n_groups = (1024 + pairs - 1) / pairs;
            if (n_groups > full_chunks) n_groups = full_chunks;
            c = n_groups <= 1 ? n_chunks : (int)((full_chunks + n_groups - 1) / n_groups);
        }
        if (c > n_chunks) c = n_chunks;
        if (c < 1) c = 1;
    }
    *n_waves = w;
    *chunks_per_group = c;
}

}  // namespace

int pz::launch_override(int which) {
    return (which >= 0 && which < PZ_OVERRIDE_COUNT) ? g_override[which].load(std::memory_order_relaxed) : -1;
}

extern "C" {

pz_status pz_debug_set_launch_override(int32_t which, int32_t value) {
    if (which < 0 || which >= PZ_OVERRIDE_COUNT) return PZ_ERR_SHAPE;
    const bool counts = which == PZ_OVERRIDE_ATTN_WAVES || which == PZ_OVERRIDE_ATTN_CHUNKS_PER_GROUP;
    if (!counts && value > 1) return PZ_ERR_SHAPE;
    g_override[which].store((value < 0 || (counts && value == 0)) ? -1 : value, std::memory_order_relaxed);
    return PZ_OK;
}

const char *pz_status_string(pz_status s) {
    switch (s) {
        case PZ_OK: return "PZ_OK";
        case PZ_ERR_NULL: return "PZ_ERR_NULL: a required pointer is NULL";
        case PZ_ERR_SHAPE: return "PZ_ERR_SHAPE: negative or inconsistent sizes";
        case PZ_ERR_UNSUPPORTED: return "PZ_ERR_UNSUPPORTED: outside the supported shapes/dtypes";
        case PZ_ERR_WORKSPACE: return "PZ_ERR_WORKSPACE: workspace missing or too small";
        case PZ_ERR_LAUNCH: return "PZ_ERR_LAUNCH: the HIP runtime refused the launch";
    }
    return "unknown pz_status";
}

pz_status pz_kv_append_fp8(const pz_cache *cache, const void *k_new, const void *v_new,
                           const int64_t *slot_mapping, int64_t n_tokens, float k_scale,
                           float v_scale, void *hip_stream) {
    const pz_status cs = check_cache(cache, true);
    if (cs != PZ_OK) return cs;
    if (n_tokens < 0) return PZ_ERR_SHAPE;
    if (n_tokens == 0) return PZ_OK;
    if (k_new == nullptr || v_new == nullptr || slot_mapping == nullptr) return PZ_ERR_NULL;
    if (cache->n_kv_heads > 65535) return PZ_ERR_UNSUPPORTED;
    if (cache->dtype == PZ_KV_FP8_E4M3 && (!positive_finite(k_scale) || !positive_finite(v_scale)))
        return PZ_ERR_SHAPE;
    pz::AppendParams p;
    p.k = static_cast<uint8_t *>(cache->k);
    p.v = static_cast<uint8_t *>(cache->v);
    p.k_new = static_cast<const uint16_t *>(k_new);
    p.v_new = static_cast<const uint16_t *>(v_new);
    p.slot_mapping = slot_mapping;
    p.T = n_tokens;
    p.Hkv = cache->n_kv_heads;
    p.P = cache->page_size;
    p.D = cache->head_dim;
    p.num_slots = cache->num_pages * (int64_t)cache->page_size;
    p.k_scale = k_scale;
    p.v_scale = v_scale;
    const hipError_t e = pz::launch_kv_append(p, cache->dtype == PZ_KV_FP8_E4M3 ? 1 : 2,
                                              static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? PZ_OK : PZ_ERR_LAUNCH;
}

int32_t pz_decode_attn_n_splits(int32_t max_seq_len, int32_t window, int32_t split_tokens) {
    if (max_seq_len < 0 || window < 0 || split_tokens <= 0 || split_tokens % 64 != 0) return 0;
    int64_t span = max_seq_len;
    if (window > 0 && (int64_t)window + 63 < span) span = (int64_t)window + 63;
    const int64_t n = (span + split_tokens - 1) / split_tokens;
    return (int32_t)(n < 1 ? 1 : n);
}

size_t pz_decode_attn_workspace_bytes(int32_t batch, int32_t n_q_heads, int32_t head_dim,
                                      int32_t n_splits) {
    if (batch <= 0 || n_q_heads <= 0 || head_dim <= 0 || n_splits <= 0) return 0;
    return (size_t)batch * (size_t)n_q_heads * (size_t)n_splits * (size_t)(head_dim + 2) * sizeof(float);
}

namespace {

pz_status decode_attn_impl(const pz_cache *cache, const void *k_new, const void *v_new, bool fused_append,
                           const void *q, const int32_t *block_table,
                           int32_t max_pages_per_seq, const int32_t *seq_lens, int32_t batch,
                           int32_t n_q_heads, const float *sinks, float sm_scale, float k_scale,
                           float v_scale, int32_t window, int32_t split_tokens, int32_t n_splits,
                           void *workspace, size_t workspace_bytes, void *out, int32_t out_dtype,
                           void *hip_stream) {
    const pz_status cs = check_cache(cache, true);
    if (cs != PZ_OK) return cs;
    const bool wide = cache->head_dim == 128;
    if (batch < 0 || n_q_heads <= 0 || max_pages_per_seq <= 0 || window < 0 || split_tokens < 0)
        return PZ_ERR_SHAPE;
    if (n_q_heads % cache->n_kv_heads != 0) return PZ_ERR_SHAPE;
    if (!group_supported(n_q_heads / cache->n_kv_heads)) return PZ_ERR_UNSUPPORTED;
    if ((int64_t)max_pages_per_seq * cache->page_size > kMaxPositions) return PZ_ERR_UNSUPPORTED;
    if (out_dtype != PZ_OUT_F32 && out_dtype != PZ_OUT_BF16) return PZ_ERR_UNSUPPORTED;
    if (!positive_finite(sm_scale) || !positive_finite(k_scale) || !positive_finite(v_scale))
        return PZ_ERR_SHAPE;
    if (split_tokens % 64 != 0) return PZ_ERR_UNSUPPORTED;
    if (batch == 0) return PZ_OK;
    if (q == nullptr || block_table == nullptr || seq_lens == nullptr) return PZ_ERR_NULL;
    if (fused_append && (k_new == nullptr || v_new == nullptr)) return PZ_ERR_NULL;
    if (split_tokens > 0) {
        if (n_splits <= 0) return PZ_ERR_SHAPE;
        if ((int64_t)n_splits * split_tokens > 0x7fffffffLL) return PZ_ERR_UNSUPPORTED;   // positions are 32-bit
        if (workspace == nullptr) return PZ_ERR_WORKSPACE;
        if (workspace_bytes < pz_decode_attn_workspace_bytes(batch, n_q_heads, cache->head_dim, n_splits))
            return PZ_ERR_WORKSPACE;
    } else if (out == nullptr) {
        return PZ_ERR_NULL;
    }
    const int n_chunks = split_tokens > 0 ? n_splits : 1;
    if ((int64_t)batch * cache->n_kv_heads * 8 * n_chunks > 0x7fffffffLL) return PZ_ERR_UNSUPPORTED;

    pz::AttnParams p;
    p.k = static_cast<uint8_t *>(cache->k);
    p.v = static_cast<uint8_t *>(cache->v);
    // The fused append runs inside the attention launch: the wave that attends the newest position takes it
    // from k_new / v_new in registers, behind its step loop, and writes the cache bytes when it is done (batch
    // 16 x 64K: 2 to 3 us less per step than with an append launch, batch 64 x 8K 2.4, batch 256 at window
    // 128: 1.3).  Above 1024 (sequence, KV head) pairs in a split-K call it gets a launch of its own first
    // instead: there every wave carries the extra round trip at its end and 64 scattered V bytes, which
    // together cost more than the launch (batch 256 at window 8192: + 13 us of 338).  Same bytes either way.
    bool in_kernel = fused_append && (split_tokens == 0 || (int64_t)batch * cache->n_kv_heads <= 1024);
    if (fused_append && pz::launch_override(PZ_OVERRIDE_APPEND_FUSED) >= 0)
        in_kernel = pz::launch_override(PZ_OVERRIDE_APPEND_FUSED) == 1;
    if (cache->n_kv_heads > 65535) in_kernel = fused_append;      // the append launch has one grid row per KV head
    if (wide) {                                                   // 128-channel heads: always a launch of its own
        if (fused_append && cache->n_kv_heads > 65535) return PZ_ERR_UNSUPPORTED;
        in_kernel = false;
    }
    p.k_new = in_kernel ? static_cast<const uint16_t *>(k_new) : nullptr;
    p.v_new = in_kernel ? static_cast<const uint16_t *>(v_new) : nullptr;
    p.k_scale = k_scale;
    p.q = static_cast<const uint16_t *>(q);
    p.block_table = block_table;
    p.seq_lens = seq_lens;
    p.sinks = sinks;
    p.ws_acc = static_cast<float *>(workspace);
    p.ws_ml = split_tokens > 0
                  ? static_cast<float *>(workspace) + (size_t)batch * n_q_heads * n_splits * cache->head_dim
                  : nullptr;
    p.out = out;
    p.max_pages = max_pages_per_seq;
    p.num_pages = (int32_t)cache->num_pages;
    p.max_len = max_pages_per_seq * cache->page_size;
    p.B = batch;
    p.Hq = n_q_heads;
    p.cache_heads = cache->n_kv_heads;
    p.head_shift = group_shift(n_q_heads / cache->n_kv_heads);
    p.Hkv = cache->n_kv_heads << p.head_shift;
    p.G_full = n_q_heads / cache->n_kv_heads;
    p.G = (p.G_full + (1 << p.head_shift) - 1) >> p.head_shift;
    p.window = window;
    p.split_tokens = split_tokens;
    p.n_splits = split_tokens > 0 ? n_splits : 1;
    p.out_dtype = out_dtype;
    p.sc = sm_scale * k_scale * 1.4426950408889634f;
    p.v_scale = v_scale;

    // upper bound of the 64-position steps one workgroup may see
    int64_t max_tokens = (int64_t)max_pages_per_seq * cache->page_size;
    if (window > 0 && (int64_t)window + 63 < max_tokens) max_tokens = (int64_t)window + 63;
    if (split_tokens > 0 && split_tokens < max_tokens) max_tokens = split_tokens;
    const int max_steps = (int)((max_tokens + 63) / 64);
    int n_waves = 1, chunks_per_group = 1;
    // whole chunks of the longest sequence a call can hold (a window's last chunk has at most 63 positions)
    int full_chunks = n_chunks;
    if (window > 0 && split_tokens > 0) {
        full_chunks = window / split_tokens;
        full_chunks = full_chunks < 1 ? 1 : (full_chunks > n_chunks ? n_chunks : full_chunks);
    }
    pick_shape(batch, p.Hkv, max_steps, n_chunks, full_chunks, &n_waves, &chunks_per_group);
    if (wide && n_waves > 1) {                                    // one-wave workgroups only: one chunk each then
        n_waves = 1;
        chunks_per_group = 1;
    }
    p.chunks_per_group = chunks_per_group;
    const int elem_bytes = cache->dtype == PZ_KV_FP8_E4M3 ? 1 : 2;
    hipError_t e;
    if (fused_append && !in_kernel) {
        pz::AppendParams a;
        a.k = p.k;
        a.v = p.v;
        a.k_new = static_cast<const uint16_t *>(k_new);
        a.v_new = static_cast<const uint16_t *>(v_new);
        a.slot_mapping = nullptr;
        a.T = batch;
        a.Hkv = cache->n_kv_heads;
        a.P = cache->page_size;
        a.D = cache->head_dim;
        a.num_slots = cache->num_pages * (int64_t)cache->page_size;
        a.k_scale = k_scale;
        a.v_scale = v_scale;
        e = pz::launch_kv_append_last(a, block_table, max_pages_per_seq, seq_lens, batch, elem_bytes,
                                      static_cast<hipStream_t>(hip_stream));
        if (e != hipSuccess) return PZ_ERR_LAUNCH;
    }
    // Full-attention split-K with one-wave workgroups: the chunks are dealt out evenly on the device from
    // the actual lengths (the balanced-partition override keeps the one-workgroup-per-chunk-group grid, for
    // comparisons).  Window layers keep that grid: their sequences all span about the window, their
    // first and last chunks are short, which a partition by chunk count does not see, and a share that
    // crosses from one short sequence into the next starts its pipeline anew each time (batch 256,
    // window 8192: 373 us on the balanced partition against 355 us on the grid).
    if (wide)
        e = pz::launch_decode_attn_d128(p, cache->page_size, elem_bytes, static_cast<hipStream_t>(hip_stream));
    else if (split_tokens > 0 && window == 0 && n_waves == 1 && pz::launch_override(PZ_OVERRIDE_ATTN_BALANCED) != 0)
        e = pz::launch_decode_attn_balanced(p, cache->page_size, elem_bytes, static_cast<hipStream_t>(hip_stream));
    else
        e = pz::launch_decode_attn(p, cache->page_size, elem_bytes, n_waves, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? PZ_OK : PZ_ERR_LAUNCH;
}

}  // namespace

pz_status pz_decode_attn(const pz_cache *cache, const void *q, const int32_t *block_table,
                         int32_t max_pages_per_seq, const int32_t *seq_lens, int32_t batch,
                         int32_t n_q_heads, const float *sinks, float sm_scale, float k_scale,
                         float v_scale, int32_t window, int32_t split_tokens, int32_t n_splits,
                         void *workspace, size_t workspace_bytes, void *out, int32_t out_dtype,
                         void *hip_stream) {
    return decode_attn_impl(cache, nullptr, nullptr, false, q, block_table, max_pages_per_seq, seq_lens, batch,
                            n_q_heads, sinks, sm_scale, k_scale, v_scale, window, split_tokens, n_splits, workspace,
                            workspace_bytes, out, out_dtype, hip_stream);
}

pz_status pz_decode_attn_append(const pz_cache *cache, const void *k_new, const void *v_new, const void *q,
                                const int32_t *block_table, int32_t max_pages_per_seq, const int32_t *seq_lens,
                                int32_t batch, int32_t n_q_heads, const float *sinks, float sm_scale,
                                float k_scale, float v_scale, int32_t window, int32_t split_tokens,
                                int32_t n_splits, void *workspace, size_t workspace_bytes, void *out,
                                int32_t out_dtype, void *hip_stream) {
    return decode_attn_impl(cache, k_new, v_new, true, q, block_table, max_pages_per_seq, seq_lens, batch,
                            n_q_heads, sinks, sm_scale, k_scale, v_scale, window, split_tokens, n_splits, workspace,
                            workspace_bytes, out, out_dtype, hip_stream);
}

pz_status pz_decode_attn_splitk_reduce(const void *workspace, size_t workspace_bytes, int32_t batch,
                                       int32_t n_q_heads, int32_t head_dim, int32_t n_splits,
                                       const int32_t *seq_lens, int32_t window, int32_t split_tokens,
                                       const float *sinks, float v_scale, void *out, int32_t out_dtype,
                                       void *hip_stream) {
    if (batch < 0 || n_q_heads <= 0 || head_dim <= 0 || n_splits <= 0 || window < 0) return PZ_ERR_SHAPE;
    if (head_dim != 64 && head_dim != 128) return PZ_ERR_UNSUPPORTED;
    if (out_dtype != PZ_OUT_F32 && out_dtype != PZ_OUT_BF16) return PZ_ERR_UNSUPPORTED;
    if (seq_lens != nullptr && (split_tokens <= 0 || split_tokens % 64 != 0)) return PZ_ERR_SHAPE;
    if (seq_lens != nullptr && split_tokens > kMaxPositions) return PZ_ERR_UNSUPPORTED;
    if (!positive_finite(v_scale)) return PZ_ERR_SHAPE;
    if (batch == 0) return PZ_OK;
    if (workspace == nullptr) return PZ_ERR_WORKSPACE;
    if (workspace_bytes < pz_decode_attn_workspace_bytes(batch, n_q_heads, head_dim, n_splits))
        return PZ_ERR_WORKSPACE;
    if (out == nullptr) return PZ_ERR_NULL;
    if ((int64_t)batch * n_q_heads > 0x7fffffffLL) return PZ_ERR_UNSUPPORTED;
    pz::ReduceParams p;
    p.ws_acc = static_cast<const float *>(workspace);
    p.ws_ml = static_cast<const float *>(workspace) + (size_t)batch * n_q_heads * n_splits * head_dim;
    p.seq_lens = seq_lens;
    p.sinks = sinks;
    p.out = out;
    p.B = batch;
    p.Hq = n_q_heads;
    p.n_splits = n_splits;
    p.window = window;
    p.split_tokens = split_tokens;
    p.out_dtype = out_dtype;
    p.head_dim = head_dim;
    p.v_scale = v_scale;
    const hipError_t e = pz::launch_splitk_reduce(p, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? PZ_OK : PZ_ERR_LAUNCH;
}

}  // extern "C"

// ---- the entry point that allocates nothing -------------------------------------------------------------
// Split-K workspace of pz_decode_attn_noalloc: a device array of the library itself, one copy per GPU,
// held from the moment the code object is loaded on that GPU until the process ends.
static __device__ __align__(256) unsigned char scratch[PZ_NOALLOC_WORKSPACE_BYTES];

namespace {

constexpr int kMaxDevices = 64;
// address of `scratch` on each device, resolved at the first call with that device current (the array's
// name is only a host-side handle: kernels are given this pointer)
std::atomic<void *> g_scratch_ptr[kMaxDevices];

pz_status scratch_of_current_device(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PZ_ERR_LAUNCH;
    void *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return PZ_ERR_LAUNCH;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);      // two threads resolve the same address
    }
    *out = ptr;
    return PZ_OK;
}

}  // namespace

extern "C" {

pz_status pz_decode_attn_noalloc(const pz_cache *cache, const void *q, const int32_t *block_table,
                                 int32_t max_pages_per_seq, const int32_t *seq_lens, int32_t batch,
                                 int32_t n_q_heads, const float *sinks, float sm_scale, float k_scale,
                                 float v_scale, int32_t window, int32_t split_tokens, int32_t n_splits, void *out,
                                 int32_t out_dtype, void *hip_stream) {
    if (out == nullptr && batch > 0) return PZ_ERR_NULL;
    if (split_tokens <= 0)                              // single pass: no scratch at all
        return decode_attn_impl(cache, nullptr, nullptr, false, q, block_table, max_pages_per_seq, seq_lens, batch,
                                n_q_heads, sinks, sm_scale, k_scale, v_scale, window, split_tokens, 0, nullptr, 0, out,
                                out_dtype, hip_stream);
    if (batch < 0 || n_q_heads <= 0 || n_splits <= 0) return PZ_ERR_SHAPE;
    if (batch == 0) return PZ_OK;
    if (cache == nullptr) return PZ_ERR_NULL;
    // the partials of the call must fit the array: refused here, before anything is enqueued
    if ((uint64_t)batch * (uint64_t)n_q_heads * (uint64_t)n_splits > PZ_NOALLOC_WORKSPACE_BYTES / ((64 + 2) * sizeof(float)))
        return PZ_ERR_WORKSPACE;
    const size_t need = pz_decode_attn_workspace_bytes(batch, n_q_heads, cache->head_dim, n_splits);
    if (need == 0 || need > (size_t)PZ_NOALLOC_WORKSPACE_BYTES) return PZ_ERR_WORKSPACE;
    void *ws = nullptr;
    const pz_status ss = scratch_of_current_device(&ws);
    if (ss != PZ_OK) return ss;
    // Nothing of the array has to start at zero: the first pass writes every row that the merge uses (the
    // rows of the chunks that hold attended positions of a sequence), the merge bounds itself by the same
    // lengths, and what the array keeps from an earlier call in its other rows is fetched at most as padding
    // of a batch of loads and dropped by a select.
    const pz_status s1 = decode_attn_impl(cache, nullptr, nullptr, false, q, block_table, max_pages_per_seq, seq_lens,
                                          batch, n_q_heads, sinks, sm_scale, k_scale, v_scale, window, split_tokens,
                                          n_splits, ws, need, nullptr, out_dtype, hip_stream);
    if (s1 != PZ_OK) return s1;
    return pz_decode_attn_splitk_reduce(ws, need, batch, n_q_heads, cache->head_dim, n_splits, seq_lens, window,
                                        split_tokens, sinks, v_scale, out, out_dtype, hip_stream);
}

pz_status pz_prefill_attn(const pz_cache *cache, const void *q, const int32_t *q_start,
                          const int32_t *block_table, int32_t max_pages_per_seq, const int32_t *seq_lens,
                          int32_t batch, int32_t n_q_heads, int32_t max_new_tokens, const float *sinks,
                          float sm_scale, float k_scale, float v_scale, int32_t window, void *out,
                          int32_t out_dtype, void *hip_stream) {
    const pz_status cs = check_cache(cache);
    if (cs != PZ_OK) return cs;
    if (batch < 0 || n_q_heads <= 0 || max_pages_per_seq <= 0 || window < 0 || max_new_tokens < 0) return PZ_ERR_SHAPE;
    if (n_q_heads % cache->n_kv_heads != 0) return PZ_ERR_SHAPE;
    if (!group_supported(n_q_heads / cache->n_kv_heads)) return PZ_ERR_UNSUPPORTED;
    if ((int64_t)max_pages_per_seq * cache->page_size > kMaxPositions) return PZ_ERR_UNSUPPORTED;
    if (out_dtype != PZ_OUT_F32 && out_dtype != PZ_OUT_BF16) return PZ_ERR_UNSUPPORTED;
    if (!positive_finite(sm_scale) || !positive_finite(k_scale) || !positive_finite(v_scale)) return PZ_ERR_SHAPE;
    if (batch == 0 || max_new_tokens == 0) return PZ_OK;
    if (q == nullptr || q_start == nullptr || block_table == nullptr || seq_lens == nullptr || out == nullptr)
        return PZ_ERR_NULL;
    const int tiles = (max_new_tokens + 2 * PZ_PREFILL_NT - 1) / (2 * PZ_PREFILL_NT);
    if ((int64_t)batch * tiles * cache->n_kv_heads * 8 > 0x7fffffffLL) return PZ_ERR_UNSUPPORTED;
    pz::PrefillParams p;
    p.k = static_cast<const uint8_t *>(cache->k);
    p.v = static_cast<const uint8_t *>(cache->v);
    p.q = static_cast<const uint16_t *>(q);
    p.q_start = q_start;
    p.block_table = block_table;
    p.seq_lens = seq_lens;
    p.sinks = sinks;
    p.out = out;
    p.max_pages = max_pages_per_seq;
    p.num_pages = (int32_t)cache->num_pages;
    p.max_len = max_pages_per_seq * cache->page_size;
    p.B = batch;
    p.Hq = n_q_heads;
    p.cache_heads = cache->n_kv_heads;
    p.head_shift = group_shift(n_q_heads / cache->n_kv_heads);
    p.Hkv = cache->n_kv_heads << p.head_shift;
    p.G_full = n_q_heads / cache->n_kv_heads;
    p.G = (p.G_full + (1 << p.head_shift) - 1) >> p.head_shift;
    p.window = window;
    p.out_dtype = out_dtype;
    p.tiles_per_seq = tiles;
    p.sc = sm_scale * k_scale * 1.4426950408889634f;
    p.v_scale = v_scale;
    const hipError_t e = pz::launch_prefill_attn(p, cache->page_size, cache->dtype == PZ_KV_FP8_E4M3 ? 1 : 2, tiles,
                                                 static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? PZ_OK : PZ_ERR_LAUNCH;
}

pz_status pz_rope_yarn_table(const pz_yarn_params *prm, int32_t head_dim, int32_t n_pos, float *cos_out,
                             float *sin_out) {
    if (prm == nullptr || cos_out == nullptr || sin_out == nullptr) return PZ_ERR_NULL;
    if (head_dim <= 0 || head_dim % 2 != 0 || n_pos < 0 || prm->original_context <= 0) return PZ_ERR_SHAPE;
    if (!(prm->theta > 1.0f) || !(prm->factor >= 1.0f) || !(prm->beta_fast > prm->beta_slow) || !(prm->beta_slow > 0.0f))
        return PZ_ERR_SHAPE;
    const int half = head_dim / 2;
    const double two_pi = 6.283185307179586476925286766559;
    // dimension (fractional) whose wavelength completes `rot` rotations over the original context
    auto corr_dim = [&](double rot) {
        return head_dim * log(prm->original_context / (rot * two_pi)) / (2.0 * log((double)prm->theta));
    };
    const double low = corr_dim(prm->beta_fast), high = corr_dim(prm->beta_slow);
    const double temperature = prm->factor > 1.0f ? 0.1 * log((double)prm->factor) + 1.0 : 1.0;
    for (int i = 0; i < half; ++i) {
        const double freq = pow((double)prm->theta, -2.0 * i / head_dim);      // extrapolation
        double ramp = (i - low) / (high - low);
        ramp = ramp < 0.0 ? 0.0 : (ramp > 1.0 ? 1.0 : ramp);                    // 0: keep, 1: interpolate
        const double inv = freq * (1.0 - ramp) + (freq / prm->factor) * ramp;
        for (int p = 0; p < n_pos; ++p) {
            const double ang = p * inv;
            cos_out[(size_t)p * half + i] = (float)(cos(ang) * temperature);
            sin_out[(size_t)p * half + i] = (float)(sin(ang) * temperature);
        }
    }
    return PZ_OK;
}

pz_status pz_rope_kv_append_fp8(const pz_cache *cache, const void *q_in, void *q_out, const void *k_new,
                                const void *v_new, const int32_t *positions, const float *cos_tab,
                                const float *sin_tab, const int64_t *slot_mapping, int64_t n_tokens,
                                int32_t n_q_heads, float k_scale, float v_scale, void *hip_stream) {
    const pz_status cs = check_cache(cache);
    if (cs != PZ_OK) return cs;
    if (n_tokens < 0 || n_q_heads < 0) return PZ_ERR_SHAPE;
    if (n_tokens == 0) return PZ_OK;
    if (k_new == nullptr || v_new == nullptr || slot_mapping == nullptr || positions == nullptr ||
        cos_tab == nullptr || sin_tab == nullptr)
        return PZ_ERR_NULL;
    if (n_q_heads > 0 && (q_in == nullptr || q_out == nullptr)) return PZ_ERR_NULL;
    if (cache->n_kv_heads + n_q_heads > 65535) return PZ_ERR_UNSUPPORTED;
    if (cache->dtype == PZ_KV_FP8_E4M3 && (!positive_finite(k_scale) || !positive_finite(v_scale)))
        return PZ_ERR_SHAPE;
    pz::RopeAppendParams p;
    p.ap.k = static_cast<uint8_t *>(cache->k);
    p.ap.v = static_cast<uint8_t *>(cache->v);
    p.ap.k_new = static_cast<const uint16_t *>(k_new);
    p.ap.v_new = static_cast<const uint16_t *>(v_new);
    p.ap.slot_mapping = slot_mapping;
    p.ap.T = n_tokens;
    p.ap.Hkv = cache->n_kv_heads;
    p.ap.P = cache->page_size;
    p.ap.D = cache->head_dim;
    p.ap.num_slots = cache->num_pages * (int64_t)cache->page_size;
    p.ap.k_scale = k_scale;
    p.ap.v_scale = v_scale;
    p.q_in = static_cast<const uint16_t *>(q_in);
    p.q_out = static_cast<uint16_t *>(q_out);
    p.positions = positions;
    p.cos_tab = cos_tab;
    p.sin_tab = sin_tab;
    p.Hq = n_q_heads;
    const hipError_t e = pz::launch_rope_kv_append(p, cache->dtype == PZ_KV_FP8_E4M3 ? 1 : 2,
                                                   static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? PZ_OK : PZ_ERR_LAUNCH;
}

pz_status pz_kv_amax_update(const void *k, const void *v, int64_t n_elems, float *amax, void *hip_stream) {
    if (n_elems < 0) return PZ_ERR_SHAPE;
    if (n_elems == 0) return PZ_OK;
    if (k == nullptr || v == nullptr || amax == nullptr) return PZ_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(k) | reinterpret_cast<uintptr_t>(v)) & 15u) return PZ_ERR_UNSUPPORTED;
    const hipError_t e = pz::launch_kv_amax(static_cast<const uint16_t *>(k), static_cast<const uint16_t *>(v),
                                            n_elems, amax, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? PZ_OK : PZ_ERR_LAUNCH;
}

pz_status pz_kv_scales_from_amax(const float *amax, int32_t round_up_pow2, float *scales, void *hip_stream) {
    if (amax == nullptr || scales == nullptr) return PZ_ERR_NULL;
    const hipError_t e = pz::launch_kv_scales(amax, round_up_pow2 != 0, scales, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? PZ_OK : PZ_ERR_LAUNCH;
}

}  // extern "C"
