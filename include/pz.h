/*
 * pz.h -- C ABI of the MI355X (gfx950) decode-attention library.
 *
 * The library implements the part of a decode step whose cost the paper's inference
 * optimisations act on: single-token grouped-query attention over a paged KV cache that is
 * stored in FP8 (E4M3) with one calibrated K scale and one V scale per layer (paper Section 3,
 * "KV Quantization"), where each layer is either full-context or sliding-window attention
 * (Section 2, "Window attention for long-context inference"), plus the kernel that quantises
 * and appends the new token's K/V to that cache.  Learned per-head attention-sink logits (a
 * property of the gpt-oss parent model) take part in the softmax denominator.
 *
 * Conventions that hold for every entry point:
 *   - Every pointer is a DEVICE pointer unless marked "host".  The pz_cache descriptor itself
 *     is a host struct (its k / v members are device pointers).
 *   - The caller owns every buffer.  The library never allocates, frees or synchronises; each
 *     call only enqueues kernels on `hip_stream` (a hipStream_t, NULL = the default stream) and
 *     returns.  Buffers must stay alive until the stream has run past the call.
 *   - Argument errors are detected on the host before anything is enqueued and are reported
 *     through the return value (never abort, never throw).  A failed launch gives
 *     PZ_ERR_LAUNCH.  What lives in device memory cannot be checked there: block-table entries,
 *     sequence lengths and slots outside their ranges are the caller's bug and are not reported.
 *     The kernels hold them to the buffers all the same -- a page id is cut to [0, num_pages), a
 *     length to max_pages_per_seq * page_size (a negative one counts as 0), and a token whose slot
 *     or page lies outside the cache is not written -- so such a sequence gets a meaningless row,
 *     every other sequence its proper one, and no access leaves the cache or the block table.
 *     (Not covered: q_start of the prefill call and positions of the rotary call, which index
 *     buffers whose sizes the calls do not take.)
 *   - Positions are 32-bit: max_pages_per_seq * page_size may not exceed 2^30 and
 *     n_splits * split_tokens must stay below 2^31 (PZ_ERR_UNSUPPORTED otherwise).
 *   - Supported shapes: head_dim == 64 (the parent model's; every entry point), or 128 for
 *     pz_kv_append_fp8, pz_decode_attn, pz_decode_attn_append (which then always appends by a launch
 *     of its own), pz_decode_attn_splitk_reduce and pz_decode_attn_noalloc -- one plain launch form,
 *     not the tuned path; pz_prefill_attn and pz_rope_kv_append_fp8 return PZ_ERR_UNSUPPORTED for it.
 *     page_size in {16, 32, 64}; n_q_heads a multiple of
 *     n_kv_heads with group size n_q_heads / n_kv_heads <= 64 (a group above 8 is cut into 2, 4
 *     or 8 parts of at most 8 heads and the attention kernels read each KV head once per part).
 *
 *   - Launch shapes are chosen by the library from the arguments alone; no environment variable is read.
 *     pz_debug_set_launch_override (below) forces a shape, for tests and measurements.
 *
 * Cache layout (chosen for the matrix-core operand shapes of gfx950; the paper does not
 * discuss paging):
 *     K : [num_pages][n_kv_heads][page_size][head_dim]     (a token's channels are contiguous)
 *     V : [num_pages][n_kv_heads][head_dim][page_size]     (a channel's tokens are contiguous)
 *   element = 1 byte OCP FP8 E4M3 (PZ_KV_FP8_E4M3) or 2 bytes bf16 (PZ_KV_BF16).
 *   A "slot" is physical_page * page_size + offset_in_page.
 */
#ifndef PZ_H
#define PZ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PZ_OK = 0,
    PZ_ERR_NULL = -1,         /* a required pointer is NULL */
    PZ_ERR_SHAPE = -2,        /* negative / inconsistent sizes */
    PZ_ERR_UNSUPPORTED = -3,  /* valid request outside the supported set above */
    PZ_ERR_WORKSPACE = -4,    /* workspace missing or too small */
    PZ_ERR_LAUNCH = -5        /* the HIP runtime refused the launch */
} pz_status;

typedef enum { PZ_KV_FP8_E4M3 = 0, PZ_KV_BF16 = 1 } pz_kv_dtype;
typedef enum { PZ_OUT_F32 = 0, PZ_OUT_BF16 = 1 } pz_out_dtype;

typedef struct {
    void *k;                  /* device, layout above */
    void *v;                  /* device, layout above */
    int32_t num_pages;
    int32_t page_size;
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t dtype;            /* pz_kv_dtype */
} pz_cache;

/* Human-readable name of a status code (host string, static storage). */
const char *pz_status_string(pz_status s);

/*
 * Test and measurement hook, not part of the decode path: forces one of the launch-shape choices the
 * library otherwise makes from the arguments of a call (results are the same for every shape; the
 * split-K workspace rows that hold partials depend on it, as stated at pz_decode_attn_workspace_bytes).
 * Process-wide, takes effect for the calls that follow; a negative value hands the choice back.
 *   PZ_OVERRIDE_ATTN_WAVES             1 | 2 | 4 | 8   waves per workgroup of the decode-attention kernel (0 = unset)
 *   PZ_OVERRIDE_ATTN_CHUNKS_PER_GROUP  n >= 1          consecutive split-K chunks walked by a one-wave workgroup (0 = unset)
 *   PZ_OVERRIDE_ATTN_BALANCED          0 | 1           0: full-attention split-K on the fixed (sequence, chunk
 *                                                      group) grid instead of the partition balanced over the batch
 *   PZ_OVERRIDE_APPEND_FORM            0 | 1           quantise-and-append as 64-token tiles (0; large appends) or
 *                                                      as one wave per (token, KV head) (1; decode-sized appends)
 *   PZ_OVERRIDE_APPEND_FUSED           0 | 1           pz_decode_attn_append appends by a launch of its own first
 *                                                      (0) or inside the attention launch (1)
 * Returns PZ_ERR_SHAPE for an unknown override or a value outside the listed ones.
 */
typedef enum {
    PZ_OVERRIDE_ATTN_WAVES = 0,
    PZ_OVERRIDE_ATTN_CHUNKS_PER_GROUP = 1,
    PZ_OVERRIDE_ATTN_BALANCED = 2,
    PZ_OVERRIDE_APPEND_FORM = 3,
    PZ_OVERRIDE_APPEND_FUSED = 4,
    PZ_OVERRIDE_COUNT = 5
} pz_launch_override;
pz_status pz_debug_set_launch_override(int32_t which, int32_t value);

/*
 * Quantise-and-append (paper Section 3, "KV Quantization": FP8 KV cache with per-layer scales).
 *
 * For every token t < n_tokens with slot = slot_mapping[t] >= 0, every KV head g and channel c:
 *     K[slot][g][c] = e4m3( float(k_new[t][g][c]) / k_scale )       (same for V with v_scale)
 * where e4m3() rounds to nearest even and saturates at +-448 (NaN stays NaN), and the division
 * is one IEEE fp32 division.  Tokens with a negative slot are skipped; all other cache bytes are
 * left untouched.  With cache->dtype == PZ_KV_BF16 the bf16 values are copied through unscaled
 * (comparison variant; the scales are ignored).
 *
 *   k_new, v_new  : bf16 [n_tokens][n_kv_heads][head_dim], contiguous
 *   slot_mapping  : int64 [n_tokens]
 *   k_scale, v_scale : > 0 (a scale of 1 is the paper's "no scales" variant; powers of two are
 *                      its final choice -- the library takes any positive value)
 * n_tokens == 0 is legal and enqueues nothing.  Two tokens with the same slot race.
 */
pz_status pz_kv_append_fp8(const pz_cache *cache /* host */, const void *k_new, const void *v_new,
                           const int64_t *slot_mapping, int64_t n_tokens, float k_scale,
                           float v_scale, void *hip_stream);

/*
 * Number of split-K chunks that cover every sequence of a call (host arithmetic only).
 * Chunk i of sequence b covers the logical positions
 *     [a_b + i*split_tokens, a_b + (i+1)*split_tokens)  intersected with  [lo_b, L_b),
 * lo_b = max(0, L_b - window) for window > 0, else 0;  a_b = lo_b rounded down to a multiple of
 * 64.  The result is ceil(span / split_tokens) with span = max_seq_len for full attention and
 * min(max_seq_len, window + 63) for window layers.  Returns 0 for invalid arguments.
 */
int32_t pz_decode_attn_n_splits(int32_t max_seq_len, int32_t window, int32_t split_tokens);

/*
 * Bytes of split-K workspace for a call:  batch * n_q_heads * n_splits * (head_dim + 2) * 4.
 * Layout: float acc[batch][n_q_heads][n_splits][head_dim], then
 *         float ml [batch][n_q_heads][n_splits][2]  = (m, l).
 * A partial is sink-free and unnormalised:  with s_j the scaled logit of position j,
 *     m = max_j s_j (natural-log units),  l = sum_j exp(s_j - m),
 *     acc[c] = sum_j exp(s_j - m) * decode(V[j][c])        (v_scale not applied),
 * an empty row is (m = -inf, l = 0) and its acc is ignored (it may hold anything).
 * Row i of a sequence holds the partial over the positions of chunks i .. i + r - 1, r >= 1, and
 * rows i + 1 .. i + r - 1 are empty: a workgroup that is given several consecutive chunks of one
 * sequence runs them as one online softmax and leaves one partial in the row of the first (which
 * chunks share a workgroup is the library's choice and depends on the batch).  The merge is the
 * same either way: pz_decode_attn_splitk_reduce combines the rows that are not empty.
 */
size_t pz_decode_attn_workspace_bytes(int32_t batch, int32_t n_q_heads, int32_t head_dim,
                                      int32_t n_splits);

/*
 * Single-token decode attention over the paged cache (the operation whose KV-cache traffic
 * dominates long-context decoding, paper Section 2 "Optimized Scenarios"; window rule from
 * Section 2 "Window attention for long-context inference": a token attends to the most recent
 * `window` positions, its own just-appended position included).
 *
 * For every sequence b < batch and query head h (KV head g = h / (n_q_heads / n_kv_heads)), over
 * the positions j in [lo_b, L_b):
 *     s_j  = (sm_scale * k_scale) * sum_c q[b][h][c] * decode(K[j][g][c])
 *     M    = max(sink_h, max_j s_j),   D = exp(sink_h - M) + sum_j exp(s_j - M)
 *     out[b][h][c] = v_scale * sum_j exp(s_j - M) * decode(V[j][g][c]) / D
 * The sink logit is in the units of s_j, joins the maximum and the denominator and has no value
 * row; sinks == NULL means no sink (plain softmax).  L_b == 0 gives a zero row.
 *
 *   q            : bf16 [batch][n_q_heads][head_dim]
 *   block_table  : int32 [batch][max_pages_per_seq]; entry p of row b is the physical page of
 *                  positions [p*page_size, (p+1)*page_size); any entry of a row may be read, but
 *                  only entries that hold attended positions are used (the others may hold
 *                  anything, e.g. -1)
 *   seq_lens     : int32 [batch], L_b, counting the token appended in this step
 *   sinks        : fp32 [n_q_heads] or NULL
 *   sm_scale, k_scale, v_scale : > 0
 *   window       : 0 = full attention, else sliding window length
 *   split_tokens : 0 = single pass: the sink is applied and `out` is written
 *                  (workspace may be NULL, n_splits is ignored);
 *                  > 0 (a multiple of 64) = split-K: only partials are written to `workspace`
 *                  (rows as defined at pz_decode_attn_workspace_bytes; the row of a chunk that
 *                  holds no attended position of its sequence is NOT written -- it keeps whatever
 *                  it held), `out` is not touched, and the caller enqueues
 *                  pz_decode_attn_splitk_reduce with the same seq_lens / window / split_tokens
 *                  on the same stream.  Positions beyond n_splits * split_tokens of a_b are
 *                  ignored, so n_splits must be at least pz_decode_attn_n_splits(max_b L_b, ...).
 *   out          : [batch][n_q_heads][head_dim], fp32 or bf16 (round to nearest even)
 */
pz_status pz_decode_attn(const pz_cache *cache /* host */, const void *q,
                         const int32_t *block_table, int32_t max_pages_per_seq,
                         const int32_t *seq_lens, int32_t batch, int32_t n_q_heads,
                         const float *sinks, float sm_scale, float k_scale, float v_scale,
                         int32_t window, int32_t split_tokens, int32_t n_splits, void *workspace,
                         size_t workspace_bytes, void *out, int32_t out_dtype, void *hip_stream);

/*
 * pz_kv_append_fp8 of one new token per sequence and pz_decode_attn in one call.  The paper's decode
 * step quantises the new token's K/V into the FP8 cache and then attends over the cache including
 * that token (Section 3, "KV Quantization"); this call does both: the same cache bytes as the two
 * separate calls, bit for bit, and the same attention.  Where it pays (single-pass calls, split-K calls of
 * up to 1024 (sequence, KV head) pairs) the append runs inside the attention launch, one launch less per
 * decode step: the wave that attends position L_b - 1 takes that position from k_new / v_new, quantised in
 * registers, folds it into its online softmax as a last step of its own and writes the cache bytes when it
 * is done -- the outputs then equal the separate calls' up to the rounding order of that one position (a
 * few 1e-5 of the output RMS).  In larger split-K calls the call enqueues an append kernel of its own first
 * (bit-identical outputs).  It needs no slot mapping either way.
 *
 *   k_new, v_new : bf16 [batch][n_kv_heads][head_dim]; row b is written to the slot of position
 *                  L_b - 1 of sequence b, i.e. block_table[b][(L_b-1)/page_size] * page_size +
 *                  (L_b-1) % page_size (so that entry of the block table must be valid), quantised
 *                  with k_scale / v_scale exactly as pz_kv_append_fp8 does (bf16 caches: copied)
 * Sequences with L_b == 0 append nothing.  Everything else, including the split-K protocol, as in
 * pz_decode_attn.  The cache must not be read or written by other work on the device while the
 * call runs (inside the call only the workgroup that attends position L_b - 1 touches its bytes).
 */
pz_status pz_decode_attn_append(const pz_cache *cache /* host */, const void *k_new, const void *v_new,
                                const void *q, const int32_t *block_table, int32_t max_pages_per_seq,
                                const int32_t *seq_lens, int32_t batch, int32_t n_q_heads,
                                const float *sinks, float sm_scale, float k_scale, float v_scale,
                                int32_t window, int32_t split_tokens, int32_t n_splits, void *workspace,
                                size_t workspace_bytes, void *out, int32_t out_dtype, void *hip_stream);

/*
 * Second pass of split-K: log-sum-exp merge of the partials, sink, normalisation.
 *     M = max(sink_h, max_i m_i);  D = exp(sink_h - M) + sum_i l_i exp(m_i - M)
 *     out[b][h][c] = v_scale * sum_i acc_i[c] exp(m_i - M) / D
 * Empty partials (m = -inf) contribute nothing; a row whose partials are all empty is 0 (also
 * without a sink -- never NaN).  With seq_lens != NULL (and the window / split_tokens of the first
 * pass) only the chunks that hold attended positions of a sequence are used -- exactly those the
 * first pass wrote; whatever the other workspace rows hold is ignored.  With seq_lens == NULL all
 * n_splits partials of every row are used, so all of them must be valid.
 */
pz_status pz_decode_attn_splitk_reduce(const void *workspace, size_t workspace_bytes, int32_t batch,
                                       int32_t n_q_heads, int32_t head_dim, int32_t n_splits,
                                       const int32_t *seq_lens, int32_t window,
                                       int32_t split_tokens, const float *sinks, float v_scale,
                                       void *out, int32_t out_dtype, void *hip_stream);

/*
 * pz_decode_attn + pz_decode_attn_splitk_reduce in one call that allocates nothing and takes no
 * workspace: for callers that can neither call hipMalloc nor bring device memory beyond the inputs and the
 * output -- code under HIP graph capture, tight serving loops, harnesses that forbid allocation.  The
 * split-K partials go to a device array that is part of the library (PZ_NOALLOC_WORKSPACE_BYTES, held on
 * every GPU the library runs on from the load of its code until the process ends); its address on the
 * current device is looked up at the first call with that device current (make that call outside a
 * capture) and kept.  Arguments and results exactly as the two calls with a workspace of
 * pz_decode_attn_workspace_bytes(batch, n_q_heads, head_dim, n_splits) bytes; `out` is written by this call.
 *   PZ_ERR_WORKSPACE   the partials of the call would not fit the array (nothing is enqueued)
 *   split_tokens == 0  single pass, no partials: the same as pz_decode_attn (n_splits ignored)
 * seq_lens is required (the merge uses only the rows this call wrote; what the array keeps from earlier
 * calls is never used, so nothing is cleared).  All calls on one GPU share the one array: calls that
 * overlap on a GPU -- different streams, different host threads -- race; calls on one stream do not.
 */
#define PZ_NOALLOC_WORKSPACE_BYTES (32u << 20)
pz_status pz_decode_attn_noalloc(const pz_cache *cache /* host */, const void *q, const int32_t *block_table,
                                 int32_t max_pages_per_seq, const int32_t *seq_lens, int32_t batch,
                                 int32_t n_q_heads, const float *sinks, float sm_scale, float k_scale,
                                 float v_scale, int32_t window, int32_t split_tokens, int32_t n_splits, void *out,
                                 int32_t out_dtype, void *hip_stream);

/*
 * Multi-token (prefill / chunked-prefill) attention over the paged cache: the input half of the
 * paper's fixed-length serving scenarios (Section 4, 4K/4K and 64K/64K input/output), with the
 * same per-layer window rule and the same FP8 cache as the decode call.
 *
 * The n_b = q_start[b+1] - q_start[b] newest positions of sequence b are queries; their K/V are
 * already in the cache (append first).  Query i of sequence b sits at position
 * p = L_b - n_b + i and attends to the positions j in [lo, p], lo = max(0, p - window + 1) for
 * window > 0, else 0, by the formula of pz_decode_attn with L := p + 1 (sink included).
 *
 *   q               : bf16 [T][n_q_heads][head_dim], T = q_start[batch]; the queries of a sequence
 *                     are contiguous and in position order
 *   q_start         : int32 [batch + 1], q_start[0] == 0, non-decreasing
 *   seq_lens        : int32 [batch], L_b counting the new tokens (L_b >= n_b)
 *   max_new_tokens  : host upper bound of max_b n_b (sizes the launch; a larger value only costs
 *                     idle workgroups)
 *   out             : [T][n_q_heads][head_dim], fp32 or bf16
 * Everything else as in pz_decode_attn.
 */
pz_status pz_prefill_attn(const pz_cache *cache /* host */, const void *q, const int32_t *q_start,
                          const int32_t *block_table, int32_t max_pages_per_seq,
                          const int32_t *seq_lens, int32_t batch, int32_t n_q_heads,
                          int32_t max_new_tokens, const float *sinks, float sm_scale, float k_scale,
                          float v_scale, int32_t window, void *out, int32_t out_dtype,
                          void *hip_stream);

/*
 * Rotary position embedding with YaRN scaling, fused with the quantise-and-append of the new
 * token (paper Section 2, last paragraph of "Window attention for long-context inference": the
 * parent's YaRN encoding is kept and its scaling factor raised from 32 to 56).
 *
 * pz_rope_yarn_table (host arithmetic, host pointers) fills cos/sin tables [n_pos][head_dim/2]:
 *   frequency i:  f_i = theta^(-2i/head_dim);  r_i = clamp((i - low) / (high - low), 0, 1) with
 *   low / high the (fractional) dimensions whose wavelength completes beta_fast / beta_slow
 *   rotations over original_context positions;  inv_i = f_i (1 - r_i) + (f_i / factor) r_i;
 *   cos[p][i] = t cos(p inv_i), sin[p][i] = t sin(p inv_i), t = 0.1 ln(factor) + 1 (1 for factor 1).
 *   factor == 1 is plain rotary embedding.  The parent model's public configuration is theta
 *   150000, original_context 4096, beta_fast 32, beta_slow 1; the paper's factor is 56.
 *
 * pz_rope_kv_append_fp8 (device pointers; cos_tab / sin_tab are device copies of such tables, or of
 * any other [n_pos][32] tables): for every token t with position p = positions[t] and every head,
 * channel pairs (i, i+32), c = cos_tab[p][i], s = sin_tab[p][i]:
 *     o[i] = fma(x[i], c, -(x[i+32] * s)),   o[i+32] = fma(x[i+32], c, x[i] * s)     (fp32)
 *   q_out[t][h] = bf16(o)  (round to nearest even; q_in == q_out is allowed; n_q_heads == 0 skips q)
 *   K[slot][g]  = e4m3(o / k_scale) from the fp32 value (bf16 cache: bf16(o));  V as in
 *   pz_kv_append_fp8 (unrotated).  positions[t] must be < n_pos of the tables (not checked).
 */
typedef struct {
    float theta;
    float factor;
    int32_t original_context;
    float beta_fast;
    float beta_slow;
} pz_yarn_params;
pz_status pz_rope_yarn_table(const pz_yarn_params *prm /* host */, int32_t head_dim, int32_t n_pos,
                             float *cos_out /* host */, float *sin_out /* host */);
pz_status pz_rope_kv_append_fp8(const pz_cache *cache /* host */, const void *q_in, void *q_out,
                                const void *k_new, const void *v_new, const int32_t *positions,
                                const float *cos_tab, const float *sin_tab, const int64_t *slot_mapping,
                                int64_t n_tokens, int32_t n_q_heads, float k_scale, float v_scale,
                                void *hip_stream);

/*
 * Max calibration of the K and V scales of a layer (paper Section 3, "KV Quantization": scales
 * computed from a dataset by max calibration, then rounded up to a power of two; "all scales are
 * below 1" on the paper's data, the library does not require it).
 *
 * pz_kv_amax_update folds one batch into the running maxima:
 *     amax[0] = max(amax[0], max_i |k[i]|),   amax[1] = max(amax[1], max_i |v[i]|)
 *   k, v   : bf16 [n_elems] each (any shape, flattened), 16-byte aligned; NaN elements are ignored
 *   amax   : device float[2]; the caller sets it to {0, 0} before the first batch
 * pz_kv_scales_from_amax turns the maxima into scales on the device:
 *     scales[i] = amax[i] / 448  (one fp32 division);  with round_up_pow2 != 0 then the smallest
 *     power of two >= that value;  amax[i] == 0 (nothing seen) gives the neutral scale 1
 *   scales : device float[2] = (k_scale, v_scale); the caller copies them to the host to pass
 *            them to pz_kv_append_fp8 / pz_decode_attn (scalar arguments)
 */
pz_status pz_kv_amax_update(const void *k, const void *v, int64_t n_elems, float *amax, void *hip_stream);
pz_status pz_kv_scales_from_amax(const float *amax, int32_t round_up_pow2, float *scales, void *hip_stream);

/*
 * Host-side page pool of one layer's cache, with page recycling for sliding-window layers (the
 * per-layer KV footprint of a window layer is bounded by its window, paper Section 2, "Window
 * attention for long-context inference"; the memory it frees is what lets a single GPU hold a
 * larger batch).  Pure host code; the pool allocates host memory in create and frees it in destroy; when host memory
 * runs out a call fails with its error value (NULL, PZ_ERR_WORKSPACE) and the pool stays as it was.
 *
 *   pz_window_pages      most physical pages one sequence of a window layer holds at any time:
 *                        (window + page_size - 2) / page_size + 1   (0 for window <= 0)
 *   pz_page_pool_create  num_pages physical pages of page_size positions; block table of
 *                        [max_seqs][max_pages_per_seq] entries indexed by logical page
 *                        (position / page_size), all -1; window == 0 = full attention (nothing is
 *                        recycled before release).  NULL on bad arguments.
 *   pz_page_pool_append  the next position of sequence `seq` (its current length): first hands
 *                        back the pages that lie entirely before the window of the grown sequence,
 *                        then opens a new page if the position starts one.  Returns the slot of
 *                        the position (>= 0; pass it to pz_kv_append_fp8), or a negative pz_status:
 *                        PZ_ERR_WORKSPACE when no page is free, PZ_ERR_SHAPE for a bad sequence id
 *                        or a full block-table row.
 *   pz_page_pool_release hands back every page of a finished sequence and resets its length.
 *   pz_page_pool_block_table   host pointer to the table (valid until destroy).
 *   pz_page_pool_drain_updates copies up to `capacity` pending block-table changes (flat index
 *                        seq * max_pages_per_seq + logical_page, new value; oldest first) for the
 *                        caller to mirror into its device table; returns how many were copied.
 *                        Entries of recycled pages become -1; the attention kernel never uses them.
 */
typedef struct pz_page_pool pz_page_pool;
int32_t pz_window_pages(int32_t window, int32_t page_size);
pz_page_pool *pz_page_pool_create(int32_t num_pages, int32_t page_size, int32_t max_seqs,
                                  int32_t max_pages_per_seq, int32_t window);
void pz_page_pool_destroy(pz_page_pool *pool);
int64_t pz_page_pool_append(pz_page_pool *pool, int32_t seq);
pz_status pz_page_pool_release(pz_page_pool *pool, int32_t seq);
int32_t pz_page_pool_seq_len(const pz_page_pool *pool, int32_t seq);
int32_t pz_page_pool_free_pages(const pz_page_pool *pool);
const int32_t *pz_page_pool_block_table(const pz_page_pool *pool);
int32_t pz_page_pool_drain_updates(pz_page_pool *pool, int32_t *index_out, int32_t *value_out, int32_t capacity);
int32_t pz_page_pool_pending_updates(const pz_page_pool *pool);

#ifdef __cplusplus
}
#endif
#endif /* PZ_H */
