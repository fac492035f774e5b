/*
 * pz_oracle.c -- plain CPU oracle for FP8-KV decode attention.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, obviously-correct definition that the GPU library is checked against.
 * It is used by tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline leg, and by
 * nothing else.  It shares no code, header, table or helper with the HIP path.
 *
 * What it computes (paper: Section 3 "KV Quantization" for the FP8 cache with per-layer K/V
 * scales, optionally powers of two; Section 2 "Window attention for long-context inference" for
 * the "most recent W tokens" rule and GQA sharing).  The paper prints no formula for attention,
 * so the attention part is the textbook definition of softmax attention written out, two-pass
 * (max, then sum), in logical token order, with:
 *   - the OCP FP8 E4M3 format (1-4-3, bias 7, no infinities, max finite 448), round to nearest
 *     even, saturating at +-448;
 *   - quantisation  code = e4m3(x / scale)  with one IEEE fp32 division, dequantisation
 *     x ~= decode(code) * scale;
 *   - a learned per-query-head sink logit that takes part in the max and in the softmax
 *     denominator and contributes no value row;
 *   - window W > 0: only the last min(W, L) cached positions are attended (the token appended
 *     in this step is one of them); W == 0: all L positions.
 *
 * Oracle cache layout (its own; NOT the GPU library's):  k_cache, v_cache are
 *   [num_slots][Hkv][d]   with slot = physical_page * P + offset_in_page,
 * element = 1 byte (E4M3) or 2 bytes (bf16 bit pattern).
 *
 * Arithmetic is fp32 (accum == 0) or fp64 (accum == 1) for the dot products, the softmax sums
 * and the PV sums; decode()/bf16 widening are exact in either.  No blocking, no fusion, no
 * reordering: every loop below runs in the order of the definition.  Build with
 * -ffp-contract=off and without fast-math so that each fp32 operation rounds once, as written.
 *
 * Max calibration of the scales (amax / 448, optional power-of-two round-up) is here as well.
 *
 * Pins (tests/test_oracle_*.py): E4M3 codec against torch.float8_e4m3fn and a nearest-value
 * search in exact arithmetic; attention against a dense float64 numpy softmax; closed forms for
 * L = 1, q = 0, equal keys; window >= L == full; sink = -inf == plain softmax; chunked partials
 * merged == unsplit; rotary tables against plain rotary embedding at factor 1 and the defining
 * properties of the YaRN blend.
 * "parity unpinned" (readings that nothing the paper prints can confirm; their tests restate the
 * reading): the sink semantics (the paper only cites sink attention; the logit-in-the-denominator
 * form is the parent model's public definition); of pzo_yarn_table everything beyond the factor
 * 56 -- the temperature 0.1 ln(factor) + 1 and the constants theta, beta_fast, beta_slow and
 * original context, which are the published YaRN rule with the parent's public configuration
 * (Section 2 gives only the change of the factor from 32 to 56); model-level accuracy effects of
 * the scales (paper Table 4), which need weights and benchmark suites that are not available.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ bf16 <-> fp32 */

float pzo_bf16_to_f32(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round-to-nearest-even fp32 -> bf16 (NaN stays NaN, quiet) */
uint16_t pzo_f32_to_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

/* ------------------------------------------------------------------ E4M3 codec */

/* decode: sign s, exponent field e (bias 7), mantissa m.
 *   e == 0        : (-1)^s * m * 2^-9            (subnormals, and +-0)
 *   0 < e         : (-1)^s * (1 + m/8) * 2^(e-7)
 *   e == 15, m==7 : NaN (the format has no infinities) */
float pzo_e4m3_decode(uint8_t c) {
    int s = c >> 7, e = (c >> 3) & 15, m = c & 7;
    if (e == 15 && m == 7) return s ? -NAN : NAN;
    float mag = (e == 0) ? ldexpf((float)m, -9) : ldexpf(1.0f + (float)m / 8.0f, e - 7);
    return s ? -mag : mag;
}

/* encode: round to nearest, ties to even mantissa; |x| > 448 (and +-inf) saturate to +-448;
 * NaN -> sign|0x7F; values that round to zero keep their sign (0x80 for negatives). */
uint8_t pzo_e4m3_encode(float x) {
    uint8_t sign = signbit(x) ? 0x80 : 0x00;
    if (isnan(x)) return sign | 0x7F;
    float a = fabsf(x);
    if (a > 448.0f) return sign | 0x7E;
    if (a < 0x1p-6f) {
        /* subnormal range: spacing 2^-9; m == 8 is the code of 2^-6, the natural carry */
        int m = (int)nearbyintf(a * 512.0f);
        return sign | (uint8_t)m;
    }
    int ex;
    (void)frexpf(a, &ex);           /* a = f * 2^ex, f in [0.5, 1) */
    int e = ex - 1;                 /* a = frac * 2^e, frac in [1, 2) */
    float frac = ldexpf(a, -e);
    int m = (int)nearbyintf((frac - 1.0f) * 8.0f);
    if (m == 8) { m = 0; e += 1; }
    int code = ((e + 7) << 3) | m;
    if (code > 0x7E) code = 0x7E;
    return sign | (uint8_t)code;
}

/* quantise one bf16 value with a per-tensor scale: one fp32 division, then encode */
uint8_t pzo_quantize(uint16_t x_bf16, float scale) {
    float r = pzo_bf16_to_f32(x_bf16) / scale;
    return pzo_e4m3_encode(r);
}

/* round a positive scale up to a power of two (paper Section 3, "KV Quantization") */
float pzo_round_scale_up_pow2(float s) {
    int ex;
    float f = frexpf(s, &ex);       /* s = f * 2^ex, f in [0.5, 1) */
    return (f == 0.5f) ? s : ldexpf(1.0f, ex);
}

/* ------------------------------------------------------------------ rotary embedding (YaRN) */

/* cos/sin tables [n_pos][d/2] of YaRN-scaled rotary embedding (the paper raises the parent's YaRN
 * factor from 32 to 56, Section 2).  Per frequency pair i: extrapolated frequency f = theta^(-2i/d),
 * interpolated frequency f / factor; the number of rotations pair i completes over the original
 * context, rot_i = L0 f / (2 pi), decides the blend: rot_i >= beta_fast keeps f, rot_i <= beta_slow
 * takes f / factor, in between the blend is linear IN THE DIMENSION INDEX between the two
 * (fractional) indices where rot equals beta_fast and beta_slow.  cos/sin carry the temperature
 * 0.1 ln(factor) + 1. */
void pzo_yarn_table(double theta, double factor, int L0, double beta_fast, double beta_slow, int d,
                    int n_pos, float *cos_out, float *sin_out) {
    const double PI = 3.14159265358979323846;
    int half = d / 2;
    /* index at which a pair completes `rot` rotations:  L0 theta^(-2i/d) / (2 pi) = rot */
    double i_fast = -log(beta_fast * 2.0 * PI / L0) / log(theta) * d / 2.0;
    double i_slow = -log(beta_slow * 2.0 * PI / L0) / log(theta) * d / 2.0;
    double t = factor > 1.0 ? 1.0 + 0.1 * log(factor) : 1.0;
    for (int i = 0; i < half; ++i) {
        double f = exp(-(2.0 * i / d) * log(theta));
        double w = (i - i_fast) / (i_slow - i_fast);       /* weight of the interpolated frequency */
        if (w < 0.0) w = 0.0;
        if (w > 1.0) w = 1.0;
        double inv = (1.0 - w) * f + w * (f / factor);
        for (int p = 0; p < n_pos; ++p) {
            cos_out[(int64_t)p * half + i] = (float)(t * cos(p * inv));
            sin_out[(int64_t)p * half + i] = (float)(t * sin(p * inv));
        }
    }
}

/* rotate one row of d bf16 channels (pairs (i, i + d/2)) by the table row of its position:
 *   o[i] = fma(x1, c, -(x2 s)),  o[i + d/2] = fma(x2, c, x1 s)   -- products and fmas round once */
static void rope_row(const uint16_t *x, const float *c, const float *s, int d, float *o) {
    int half = d / 2;
    for (int i = 0; i < half; ++i) {
        float x1 = pzo_bf16_to_f32(x[i]), x2 = pzo_bf16_to_f32(x[i + half]);
        float p1 = x2 * s[i], p2 = x1 * s[i];
        o[i] = fmaf(x1, c[i], -p1);
        o[i + half] = fmaf(x2, c[i], p2);
    }
}

/* fused rotary + append: q_out = bf16(rotated q); K code = e4m3(rotated k / k_scale) from the fp32
 * value (bf16 cache: bf16(rotated k)); V quantised unrotated.  Oracle cache layout. */
void pzo_rope_kv_append(void *k_cache, void *v_cache, int kv_dtype, int Hkv, int Hq, int d,
                        const uint16_t *q_in, uint16_t *q_out, const uint16_t *k_new,
                        const uint16_t *v_new, const int32_t *positions, const float *cos_tab,
                        const float *sin_tab, const int64_t *slot_mapping, int64_t T, float k_scale,
                        float v_scale) {
    int half = d / 2;
    float *o = (float *)malloc(sizeof(float) * (size_t)d);
    for (int64_t t = 0; t < T; ++t) {
        const float *c = cos_tab + (int64_t)positions[t] * half, *s = sin_tab + (int64_t)positions[t] * half;
        for (int h = 0; h < Hq; ++h) {
            rope_row(q_in + (t * Hq + h) * d, c, s, d, o);
            for (int i = 0; i < d; ++i) q_out[(t * Hq + h) * d + i] = pzo_f32_to_bf16(o[i]);
        }
        int64_t slot = slot_mapping[t];
        if (slot < 0) continue;
        for (int g = 0; g < Hkv; ++g) {
            rope_row(k_new + (t * Hkv + g) * d, c, s, d, o);
            for (int i = 0; i < d; ++i) {
                int64_t dst = (slot * Hkv + g) * d + i;
                if (kv_dtype == 0) {
                    ((uint8_t *)k_cache)[dst] = pzo_e4m3_encode(o[i] / k_scale);
                    ((uint8_t *)v_cache)[dst] = pzo_quantize(v_new[(t * Hkv + g) * d + i], v_scale);
                } else {
                    ((uint16_t *)k_cache)[dst] = pzo_f32_to_bf16(o[i]);
                    ((uint16_t *)v_cache)[dst] = v_new[(t * Hkv + g) * d + i];
                }
            }
        }
    }
    free(o);
}

/* ------------------------------------------------------------------ max calibration */

/* largest magnitude of a bf16 tensor; NaN elements are ignored; an empty tensor gives 0 */
float pzo_amax_bf16(const uint16_t *x, int64_t n) {
    float best = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
        float a = fabsf(pzo_bf16_to_f32(x[i]));
        if (a > best) best = a;                 /* false for NaN */
    }
    return best;
}

/* scale of max calibration (paper Section 3, "KV Quantization"): amax / 448, optionally rounded
 * up to a power of two; amax == 0 (nothing seen) gives the neutral scale 1 */
float pzo_scale_from_amax(float amax, int round_up_pow2) {
    float s = amax / 448.0f;
    if (!(s > 0.0f)) return 1.0f;
    return round_up_pow2 ? pzo_round_scale_up_pow2(s) : s;
}

/* ------------------------------------------------------------------ append */

/* kv_dtype: 0 = E4M3 (1 byte), 1 = bf16 (2 bytes, copied through unscaled).
 * k_new, v_new: bf16 bit patterns [T][Hkv][d].  slot < 0 => token skipped. */
void pzo_kv_append(void *k_cache, void *v_cache, int kv_dtype, int Hkv, int d,
                   const uint16_t *k_new, const uint16_t *v_new, const int64_t *slot_mapping,
                   int64_t T, float k_scale, float v_scale) {
    for (int64_t t = 0; t < T; ++t) {
        int64_t slot = slot_mapping[t];
        if (slot < 0) continue;
        for (int g = 0; g < Hkv; ++g)
            for (int c = 0; c < d; ++c) {
                int64_t src = (t * Hkv + g) * d + c;
                int64_t dst = (slot * Hkv + g) * d + c;
                if (kv_dtype == 0) {
                    ((uint8_t *)k_cache)[dst] = pzo_quantize(k_new[src], k_scale);
                    ((uint8_t *)v_cache)[dst] = pzo_quantize(v_new[src], v_scale);
                } else {
                    ((uint16_t *)k_cache)[dst] = k_new[src];
                    ((uint16_t *)v_cache)[dst] = v_new[src];
                }
            }
    }
}

/* ------------------------------------------------------------------ attention */

typedef struct {
    const void *k_cache, *v_cache;
    int kv_dtype, P, Hkv, d;
    const uint16_t *q;
    const int32_t *block_table;
    int max_pages;
    const int32_t *seq_lens;
    int B, Hq;
    const float *sinks;
    float sm_scale, k_scale, v_scale;
    int window;
    int accum;                  /* 0: fp32 arithmetic, 1: fp64 arithmetic */
    const int32_t *rows;        /* optional list of b*Hq+h rows to compute; NULL = all */
    int64_t n_rows;
    float *out;                 /* [B][Hq][d]; only the listed rows are written */
    /* chunked variant (split-K definition); split_tokens == 0 => unsplit */
    int split_tokens, n_splits;
    float *part_acc;            /* [B][Hq][S][d] */
    float *part_ml;             /* [B][Hq][S][2] = (m, l) */
} attn_args;

static inline float cache_elem(const void *cache, int kv_dtype, int64_t idx) {
    return kv_dtype == 0 ? pzo_e4m3_decode(((const uint8_t *)cache)[idx])
                         : pzo_bf16_to_f32(((const uint16_t *)cache)[idx]);
}

/* physical slot of logical position j of sequence b */
static inline int64_t slot_of(const attn_args *a, int b, int64_t j) {
    int64_t page = a->block_table[(int64_t)b * a->max_pages + j / a->P];
    return page * a->P + j % a->P;
}

static inline int64_t window_lo(int64_t L, int window) {
    return (window > 0 && L > window) ? L - window : 0;
}

/* s_j = (sm_scale * k_scale) * sum_c q[c] * dec(K[j][c]), accumulated in channel order */
static float score_f32(const attn_args *a, int b, int h, int64_t j) {
    int g = h / (a->Hq / a->Hkv);
    float ck = a->sm_scale * a->k_scale;
    const uint16_t *qrow = a->q + ((int64_t)b * a->Hq + h) * a->d;
    int64_t base = (slot_of(a, b, j) * a->Hkv + g) * a->d;
    float acc = 0.0f;
    for (int c = 0; c < a->d; ++c) {
        float prod = pzo_bf16_to_f32(qrow[c]) * cache_elem(a->k_cache, a->kv_dtype, base + c);
        acc = acc + prod;
    }
    return ck * acc;
}

static double score_f64(const attn_args *a, int b, int h, int64_t j) {
    int g = h / (a->Hq / a->Hkv);
    double ck = (double)a->sm_scale * (double)a->k_scale;
    const uint16_t *qrow = a->q + ((int64_t)b * a->Hq + h) * a->d;
    int64_t base = (slot_of(a, b, j) * a->Hkv + g) * a->d;
    double acc = 0.0;
    for (int c = 0; c < a->d; ++c)
        acc += (double)pzo_bf16_to_f32(qrow[c]) * (double)cache_elem(a->k_cache, a->kv_dtype, base + c);
    return ck * acc;
}

/* one (b, h) row of the unsplit definition, fp32 arithmetic */
static void row_f32(const attn_args *a, int b, int h) {
    int d = a->d, g = h / (a->Hq / a->Hkv);
    float *o = a->out + ((int64_t)b * a->Hq + h) * d;
    int64_t L = a->seq_lens[b];
    for (int c = 0; c < d; ++c) o[c] = 0.0f;
    if (L <= 0) return;
    int64_t lo = window_lo(L, a->window), n = L - lo;
    float sink = a->sinks ? a->sinks[h] : -INFINITY;
    float *s = (float *)malloc(sizeof(float) * (size_t)n);
    float M = sink;
    for (int64_t j = lo; j < L; ++j) {
        s[j - lo] = score_f32(a, b, h, j);
        if (s[j - lo] > M) M = s[j - lo];
    }
    float D = expf(sink - M);           /* exp(-inf) == 0 when there is no sink */
    float *acc = (float *)calloc((size_t)d, sizeof(float));
    for (int64_t j = lo; j < L; ++j) {
        float p = expf(s[j - lo] - M);
        D = D + p;
        int64_t base = (slot_of(a, b, j) * a->Hkv + g) * d;
        for (int c = 0; c < d; ++c) {
            float pv = p * cache_elem(a->v_cache, a->kv_dtype, base + c);
            acc[c] = acc[c] + pv;
        }
    }
    for (int c = 0; c < d; ++c) o[c] = a->v_scale * acc[c] / D;
    free(acc);
    free(s);
}

/* the same row in fp64 arithmetic (error-bar reference) */
static void row_f64(const attn_args *a, int b, int h) {
    int d = a->d, g = h / (a->Hq / a->Hkv);
    float *o = a->out + ((int64_t)b * a->Hq + h) * d;
    int64_t L = a->seq_lens[b];
    for (int c = 0; c < d; ++c) o[c] = 0.0f;
    if (L <= 0) return;
    int64_t lo = window_lo(L, a->window), n = L - lo;
    double sink = a->sinks ? (double)a->sinks[h] : -INFINITY;
    double *s = (double *)malloc(sizeof(double) * (size_t)n);
    double M = sink;
    for (int64_t j = lo; j < L; ++j) {
        s[j - lo] = score_f64(a, b, h, j);
        if (s[j - lo] > M) M = s[j - lo];
    }
    double D = exp(sink - M);
    double *acc = (double *)calloc((size_t)d, sizeof(double));
    for (int64_t j = lo; j < L; ++j) {
        double p = exp(s[j - lo] - M);
        D += p;
        int64_t base = (slot_of(a, b, j) * a->Hkv + g) * d;
        for (int c = 0; c < d; ++c) acc[c] += p * (double)cache_elem(a->v_cache, a->kv_dtype, base + c);
    }
    for (int c = 0; c < d; ++c) o[c] = (float)((double)a->v_scale * acc[c] / D);
    free(acc);
    free(s);
}

/* chunked definition: chunk i of sequence b covers logical positions
 *   [a_b + i*split_tokens, a_b + (i+1)*split_tokens)  intersected with  [lo_b, L_b),
 * where a_b = lo_b rounded down to a multiple of 64.  Per chunk, sink-free and unnormalised:
 *   m = max_j s_j,  l = sum_j exp(s_j - m),  acc[c] = sum_j exp(s_j - m) * dec(V[j][c]).
 * An empty chunk is (m = -inf, l = 0, acc = 0). */
static void row_partials(const attn_args *a, int b, int h) {
    int d = a->d, g = h / (a->Hq / a->Hkv), S = a->n_splits;
    int64_t L = a->seq_lens[b];
    int64_t lo = (L > 0) ? window_lo(L, a->window) : 0;
    int64_t a0 = lo - lo % 64;
    for (int i = 0; i < S; ++i) {
        float *acc = a->part_acc + (((int64_t)b * a->Hq + h) * S + i) * d;
        float *ml = a->part_ml + (((int64_t)b * a->Hq + h) * S + i) * 2;
        for (int c = 0; c < d; ++c) acc[c] = 0.0f;
        ml[0] = -INFINITY;
        ml[1] = 0.0f;
        int64_t j0 = a0 + (int64_t)i * a->split_tokens, j1 = j0 + a->split_tokens;
        if (j0 < lo) j0 = lo;
        if (j1 > L) j1 = L;
        if (j0 >= j1) continue;
        if (a->accum == 0) {
            float m = -INFINITY, l = 0.0f;
            for (int64_t j = j0; j < j1; ++j) { float s = score_f32(a, b, h, j); if (s > m) m = s; }
            for (int64_t j = j0; j < j1; ++j) {
                float p = expf(score_f32(a, b, h, j) - m);
                l = l + p;
                int64_t base = (slot_of(a, b, j) * a->Hkv + g) * d;
                for (int c = 0; c < d; ++c) {
                    float pv = p * cache_elem(a->v_cache, a->kv_dtype, base + c);
                    acc[c] = acc[c] + pv;
                }
            }
            ml[0] = m;
            ml[1] = l;
        } else {
            double m = -INFINITY, l = 0.0;
            double *acc64 = (double *)calloc((size_t)d, sizeof(double));
            for (int64_t j = j0; j < j1; ++j) { double s = score_f64(a, b, h, j); if (s > m) m = s; }
            for (int64_t j = j0; j < j1; ++j) {
                double p = exp(score_f64(a, b, h, j) - m);
                l += p;
                int64_t base = (slot_of(a, b, j) * a->Hkv + g) * d;
                for (int c = 0; c < d; ++c) acc64[c] += p * (double)cache_elem(a->v_cache, a->kv_dtype, base + c);
            }
            for (int c = 0; c < d; ++c) acc[c] = (float)acc64[c];
            ml[0] = (float)m;
            ml[1] = (float)l;
            free(acc64);
        }
    }
}

typedef struct { const attn_args *a; int tid, nthreads; } worker_arg;

static void *worker(void *p) {
    const worker_arg *w = (const worker_arg *)p;
    const attn_args *a = w->a;
    int64_t total = a->rows ? a->n_rows : (int64_t)a->B * a->Hq;
    for (int64_t r = w->tid; r < total; r += w->nthreads) {
        int64_t row = a->rows ? a->rows[r] : r;
        int b = (int)(row / a->Hq), h = (int)(row % a->Hq);
        if (a->split_tokens > 0) row_partials(a, b, h);
        else if (a->accum == 0) row_f32(a, b, h);
        else row_f64(a, b, h);
    }
    return NULL;
}

static void run_rows(const attn_args *a, int nthreads) {
    if (nthreads < 1) nthreads = 1;
    if (nthreads > 256) nthreads = 256;
    pthread_t th[256];
    worker_arg wa[256];
    for (int t = 0; t < nthreads; ++t) {
        wa[t].a = a; wa[t].tid = t; wa[t].nthreads = nthreads;
        if (t > 0) pthread_create(&th[t], NULL, worker, &wa[t]);
    }
    worker(&wa[0]);
    for (int t = 1; t < nthreads; ++t) pthread_join(th[t], NULL);
}

/* Decode attention, unsplit.  out[b][h][:] (fp32) for every row, or for the listed rows only.
 * Rows are independent; nthreads only distributes rows over host threads. */
void pzo_decode_attn(const void *k_cache, const void *v_cache, int kv_dtype, int P, int Hkv, int d,
                     const uint16_t *q, const int32_t *block_table, int max_pages,
                     const int32_t *seq_lens, int B, int Hq, const float *sinks,
                     float sm_scale, float k_scale, float v_scale, int window, int accum,
                     const int32_t *rows, int64_t n_rows, float *out, int nthreads) {
    attn_args a;
    memset(&a, 0, sizeof a);
    a.k_cache = k_cache; a.v_cache = v_cache; a.kv_dtype = kv_dtype; a.P = P; a.Hkv = Hkv; a.d = d;
    a.q = q; a.block_table = block_table; a.max_pages = max_pages; a.seq_lens = seq_lens;
    a.B = B; a.Hq = Hq; a.sinks = sinks; a.sm_scale = sm_scale; a.k_scale = k_scale;
    a.v_scale = v_scale; a.window = window; a.accum = accum; a.rows = rows; a.n_rows = n_rows;
    a.out = out;
    run_rows(&a, nthreads);
}

/* Split-K partials by the chunked definition above (sink-free, unnormalised). */
void pzo_decode_attn_partials(const void *k_cache, const void *v_cache, int kv_dtype, int P, int Hkv,
                              int d, const uint16_t *q, const int32_t *block_table, int max_pages,
                              const int32_t *seq_lens, int B, int Hq, float sm_scale, float k_scale,
                              int window, int split_tokens, int n_splits, int accum,
                              float *part_acc, float *part_ml, int nthreads) {
    attn_args a;
    memset(&a, 0, sizeof a);
    a.k_cache = k_cache; a.v_cache = v_cache; a.kv_dtype = kv_dtype; a.P = P; a.Hkv = Hkv; a.d = d;
    a.q = q; a.block_table = block_table; a.max_pages = max_pages; a.seq_lens = seq_lens;
    a.B = B; a.Hq = Hq; a.sm_scale = sm_scale; a.k_scale = k_scale; a.window = window;
    a.accum = accum; a.split_tokens = split_tokens; a.n_splits = n_splits;
    a.part_acc = part_acc; a.part_ml = part_ml;
    run_rows(&a, nthreads);
}

/* Log-sum-exp merge of sink-free partials, then sink and normalisation (fp64 inside):
 *   M = max(sink_h, max_i m_i);  D = exp(sink_h - M) + sum_i l_i exp(m_i - M);
 *   out[c] = v_scale * sum_i acc_i[c] exp(m_i - M) / D.
 * exp(-inf) is 0; if every m_i and the sink are -inf the row is 0. */
void pzo_splitk_reduce(const float *part_acc, const float *part_ml, int B, int Hq, int d, int S,
                       const float *sinks, float v_scale, float *out) {
    for (int64_t r = 0; r < (int64_t)B * Hq; ++r) {
        int h = (int)(r % Hq);
        double sink = sinks ? (double)sinks[h] : -INFINITY;
        double M = sink;
        for (int i = 0; i < S; ++i) {
            double m = part_ml[(r * S + i) * 2];
            if (m > M) M = m;
        }
        float *o = out + r * d;
        for (int c = 0; c < d; ++c) o[c] = 0.0f;
        if (M == -INFINITY) continue;
        double D = exp(sink - M);
        for (int i = 0; i < S; ++i) {
            double m = part_ml[(r * S + i) * 2], l = part_ml[(r * S + i) * 2 + 1];
            if (m == -INFINITY) continue;
            D += l * exp(m - M);
        }
        for (int c = 0; c < d; ++c) {
            double num = 0.0;
            for (int i = 0; i < S; ++i) {
                double m = part_ml[(r * S + i) * 2];
                if (m == -INFINITY) continue;
                num += (double)part_acc[(r * S + i) * d + c] * exp(m - M);
            }
            o[c] = (float)((double)v_scale * num / D);
        }
    }
}
