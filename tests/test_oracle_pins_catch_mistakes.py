"""Do the pins have teeth?  Each case below plants one plausible mistake (a dropped term, a wrong
sign or index, a swapped operand, an off-by-one) into a COPY of oracle/pz_oracle.c, compiles the
copy and runs the pin tests of that part against it in a child process: the pins must fail.  A
control run on an unmodified copy must pass, so a failure is the mistake's and not the harness's.
Everything here runs on the CPU; the real oracle is never modified."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "pz_oracle.c")
CODEC, ATTN, ROPE = "tests/test_oracle_codec.py", "tests/test_oracle_attention.py", "tests/test_oracle_rope.py"

# (name, pin file, text in the oracle, what the mistake turns it into)
MISTAKES = [
    ("decode_exponent_bias", CODEC, "ldexpf(1.0f + (float)m / 8.0f, e - 7)", "ldexpf(1.0f + (float)m / 8.0f, e - 8)"),
    ("decode_subnormal_spacing", CODEC, "ldexpf((float)m, -9)", "ldexpf((float)m, -10)"),
    ("decode_mantissa_width", CODEC, "1.0f + (float)m / 8.0f", "1.0f + (float)m / 16.0f"),
    ("encode_ties_away_from_zero", CODEC, "int m = (int)nearbyintf((frac - 1.0f) * 8.0f);",
     "int m = (int)floorf((frac - 1.0f) * 8.0f + 0.5f);"),
    ("encode_truncates", CODEC, "int m = (int)nearbyintf((frac - 1.0f) * 8.0f);", "int m = (int)((frac - 1.0f) * 8.0f);"),
    ("encode_overflow_to_nan", CODEC, "if (a > 448.0f) return sign | 0x7E;", "if (a > 448.0f) return sign | 0x7F;"),
    ("encode_saturation_threshold", CODEC, "if (a > 448.0f) return sign | 0x7E;", "if (a >= 448.0f) return sign | 0x7D;"),
    ("encode_drops_sign_of_zero", CODEC, "uint8_t sign = signbit(x) ? 0x80 : 0x00;", "uint8_t sign = (x < 0.0f) ? 0x80 : 0x00;"),
    ("encode_subnormal_threshold", CODEC, "if (a < 0x1p-6f) {", "if (a < 0x1p-7f) {"),
    ("encode_carry_lost", CODEC, "if (m == 8) { m = 0; e += 1; }", "if (m == 8) { m = 7; }"),
    ("quantize_multiplies_by_scale", CODEC, "float r = pzo_bf16_to_f32(x_bf16) / scale;", "float r = pzo_bf16_to_f32(x_bf16) * scale;"),
    ("quantize_by_reciprocal", CODEC, "float r = pzo_bf16_to_f32(x_bf16) / scale;",
     "float r = pzo_bf16_to_f32(x_bf16) * (1.0f / scale);"),
    ("bf16_rounding_truncates", CODEC, "u += 0x7fffu + lsb;", "u += 0u * lsb;"),
    ("pow2_round_down", CODEC, "return (f == 0.5f) ? s : ldexpf(1.0f, ex);", "return (f == 0.5f) ? s : ldexpf(1.0f, ex - 1);"),
    ("pow2_exact_power_doubled", CODEC, "return (f == 0.5f) ? s : ldexpf(1.0f, ex);", "return ldexpf(1.0f, ex);"),
    ("amax_keeps_sign", CODEC, "float a = fabsf(pzo_bf16_to_f32(x[i]));", "float a = pzo_bf16_to_f32(x[i]);"),
    ("calibration_range", CODEC, "float s = amax / 448.0f;", "float s = amax / 240.0f;"),
    ("append_swaps_k_and_v", ATTN, "((uint8_t *)k_cache)[dst] = pzo_quantize(k_new[src], k_scale);",
     "((uint8_t *)k_cache)[dst] = pzo_quantize(v_new[src], k_scale);"),
    ("append_uses_k_scale_for_v", ATTN, "((uint8_t *)v_cache)[dst] = pzo_quantize(v_new[src], v_scale);",
     "((uint8_t *)v_cache)[dst] = pzo_quantize(v_new[src], k_scale);"),
    ("append_head_stride", ATTN, "int64_t dst = (slot * Hkv + g) * d + c;", "int64_t dst = (slot * Hkv + (Hkv - 1 - g)) * d + c;"),
    ("append_writes_skipped_tokens", ATTN, "        if (slot < 0) continue;\n        for (int g = 0; g < Hkv; ++g)\n            for (int c = 0; c < d; ++c) {",
     "        if (slot < 0) slot = 0;\n        for (int g = 0; g < Hkv; ++g)\n            for (int c = 0; c < d; ++c) {"),
    ("paging_offset", ATTN, "return page * a->P + j % a->P;", "return page * a->P + (j + 1) % a->P;"),
    ("paging_ignores_block_table", ATTN, "int64_t page = a->block_table[(int64_t)b * a->max_pages + j / a->P];", "int64_t page = j / a->P + 0 * b;"),
    ("window_off_by_one", ATTN, "return (window > 0 && L > window) ? L - window : 0;", "return (window > 0 && L > window) ? L - window + 1 : 0;"),
    ("window_counts_from_the_start", ATTN, "int64_t lo = window_lo(L, a->window), n = L - lo;\n    float sink",
     "int64_t lo = 0, n = L - lo;\n    float sink"),
    ("gqa_head_mapping", ATTN, "int d = a->d, g = h / (a->Hq / a->Hkv);\n    float *o = a->out + ((int64_t)b * a->Hq + h) * d;\n    int64_t L = a->seq_lens[b];\n    for (int c = 0; c < d; ++c) o[c] = 0.0f;\n    if (L <= 0) return;\n    int64_t lo = window_lo(L, a->window), n = L - lo;\n    float sink",
     "int d = a->d, g = h % a->Hkv;\n    float *o = a->out + ((int64_t)b * a->Hq + h) * d;\n    int64_t L = a->seq_lens[b];\n    for (int c = 0; c < d; ++c) o[c] = 0.0f;\n    if (L <= 0) return;\n    int64_t lo = window_lo(L, a->window), n = L - lo;\n    float sink"),
    ("score_drops_k_scale", ATTN, "float ck = a->sm_scale * a->k_scale;", "float ck = a->sm_scale;"),
    ("score_drops_sm_scale", ATTN, "float ck = a->sm_scale * a->k_scale;", "float ck = a->k_scale;"),
    ("score_reverses_channels", ATTN, "float prod = pzo_bf16_to_f32(qrow[c]) * cache_elem(a->k_cache, a->kv_dtype, base + c);",
     "float prod = pzo_bf16_to_f32(qrow[a->d - 1 - c]) * cache_elem(a->k_cache, a->kv_dtype, base + c);"),
    ("sink_left_out_of_denominator", ATTN, "float D = expf(sink - M);           /* exp(-inf) == 0 when there is no sink */", "float D = 0.0f;"),
    ("sink_sign", ATTN, "float sink = a->sinks ? a->sinks[h] : -INFINITY;", "float sink = a->sinks ? -a->sinks[h] : -INFINITY;"),
    ("sink_indexed_by_kv_head", ATTN, "float sink = a->sinks ? a->sinks[h] : -INFINITY;", "float sink = a->sinks ? a->sinks[g] : -INFINITY;"),
    ("softmax_exponent_sign", ATTN, "float p = expf(s[j - lo] - M);\n        D = D + p;", "float p = expf(M - s[j - lo]);\n        D = D + p;"),
    ("output_drops_v_scale", ATTN, "for (int c = 0; c < d; ++c) o[c] = a->v_scale * acc[c] / D;", "for (int c = 0; c < d; ++c) o[c] = acc[c] / D;"),
    ("output_not_normalised", ATTN, "for (int c = 0; c < d; ++c) o[c] = a->v_scale * acc[c] / D;", "for (int c = 0; c < d; ++c) o[c] = a->v_scale * acc[c];"),
    ("pv_reads_k", ATTN, "float pv = p * cache_elem(a->v_cache, a->kv_dtype, base + c);\n            acc[c] = acc[c] + pv;\n        }\n    }\n    for (int c = 0; c < d; ++c) o[c] = a->v_scale",
     "float pv = p * cache_elem(a->k_cache, a->kv_dtype, base + c);\n            acc[c] = acc[c] + pv;\n        }\n    }\n    for (int c = 0; c < d; ++c) o[c] = a->v_scale"),
    ("chunk_origin_not_aligned", ATTN, "int64_t a0 = lo - lo % 64;", "int64_t a0 = lo;"),
    ("chunk_overlap", ATTN, "int64_t j0 = a0 + (int64_t)i * a->split_tokens, j1 = j0 + a->split_tokens;",
     "int64_t j0 = a0 + (int64_t)i * a->split_tokens, j1 = j0 + a->split_tokens + 1;"),
    ("partial_includes_no_maximum", ATTN, "float p = expf(score_f32(a, b, h, j) - m);\n                l = l + p;", "float p = expf(score_f32(a, b, h, j));\n                l = l + p;"),
    ("reduce_weight_sign", ATTN, "D += l * exp(m - M);", "D += l * exp(M - m);"),
    ("reduce_forgets_sink", ATTN, "double D = exp(sink - M);\n        for (int i = 0; i < S; ++i) {", "double D = 0.0;\n        for (int i = 0; i < S; ++i) {"),
    ("reduce_numerator_unweighted", ATTN, "num += (double)part_acc[(r * S + i) * d + c] * exp(m - M);", "num += (double)part_acc[(r * S + i) * d + c];"),
    ("reduce_drops_v_scale", ATTN, "o[c] = (float)((double)v_scale * num / D);", "o[c] = (float)(num / D);"),
    ("rope_sin_sign", ROPE, "o[i] = fmaf(x1, c[i], -p1);", "o[i] = fmaf(x1, c[i], p1);"),
    ("rope_second_half_sign", ROPE, "o[i + half] = fmaf(x2, c[i], p2);", "o[i + half] = fmaf(x2, c[i], -p2);"),
    ("rope_interleaved_pairs", ROPE, "float x1 = pzo_bf16_to_f32(x[i]), x2 = pzo_bf16_to_f32(x[i + half]);",
     "float x1 = pzo_bf16_to_f32(x[2 * (i / 2)]), x2 = pzo_bf16_to_f32(x[2 * (i / 2) + 1]);"),
    ("rope_rotates_v", ROPE, "((uint8_t *)v_cache)[dst] = pzo_quantize(v_new[(t * Hkv + g) * d + i], v_scale);",
     "((uint8_t *)v_cache)[dst] = pzo_e4m3_encode(o[i] / v_scale);"),
    ("rope_k_quantised_from_bf16", ROPE, "((uint8_t *)k_cache)[dst] = pzo_e4m3_encode(o[i] / k_scale);",
     "((uint8_t *)k_cache)[dst] = pzo_quantize(pzo_f32_to_bf16(o[i]), k_scale);"),
    ("rope_position_row", ROPE, "const float *c = cos_tab + (int64_t)positions[t] * half, *s = sin_tab + (int64_t)positions[t] * half;",
     "const float *c = cos_tab + (int64_t)t * half, *s = sin_tab + (int64_t)t * half;"),
    ("yarn_no_temperature", ROPE, "double t = factor > 1.0 ? 1.0 + 0.1 * log(factor) : 1.0;", "double t = 1.0;"),
    ("yarn_blend_reversed", ROPE, "double inv = (1.0 - w) * f + w * (f / factor);", "double inv = w * f + (1.0 - w) * (f / factor);"),
    ("yarn_multiplies_by_factor", ROPE, "double inv = (1.0 - w) * f + w * (f / factor);", "double inv = (1.0 - w) * f + w * (f * factor);"),
    ("yarn_ramp_over_frequency", ROPE, "double w = (i - i_fast) / (i_slow - i_fast);",
     "double w = (L0 * f / (2.0 * PI) - beta_fast) / (beta_slow - beta_fast);"),
    ("yarn_theta_exponent", ROPE, "double f = exp(-(2.0 * i / d) * log(theta));", "double f = exp(-(1.0 * i / d) * log(theta));"),
]


def compile_copy(tmp_dir, name, old, new):
    text = open(SRC).read()
    if old is not None:
        assert text.count(old) == 1, "the oracle no longer holds this text exactly once: %r" % old
        text = text.replace(old, new)
    src = os.path.join(tmp_dir, name + ".c")
    so = os.path.join(tmp_dir, name + ".so")
    with open(src, "w") as f:
        f.write(text)
    subprocess.check_call(["gcc", *oracle.CFLAGS, "-Wno-unused-variable", "-Wno-unused-parameter", "-Wno-unused-function",
                           "-Wno-unused-but-set-variable", "-o", so, src, "-lm", "-lpthread"])
    return so


def run_pins(lib, files):
    env = dict(os.environ, PZ_ORACLE_LIB=lib)
    return subprocess.run([sys.executable, "-m", "pytest", *files, "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"],
                          cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)


@pytest.fixture(scope="module")
def outcomes(tmp_path_factory):
    """Every copy compiled and its pins run once, a few child processes at a time."""
    tmp_dir = str(tmp_path_factory.mktemp("oracle_copies"))
    jobs = [("control", [CODEC, ATTN, ROPE], None, None)] + [(n, [f], o, w) for n, f, o, w in MISTAKES]

    def one(job):
        name, files, old, new = job
        return name, run_pins(compile_copy(tmp_dir, name, old, new), files)

    with ThreadPoolExecutor(max_workers=max(1, min(8, len(os.sched_getaffinity(0))))) as pool:
        return dict(pool.map(one, jobs))


def test_unmodified_copy_passes_every_pin(outcomes):
    r = outcomes["control"]
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name", [m[0] for m in MISTAKES])
def test_planted_mistake_is_caught(outcomes, name):
    r = outcomes[name]
    # 1 = some pin failed; a crash of the child (negative / other codes) would be caught too, but the
    # mistakes are chosen to stay in bounds, so anything else than 1 deserves a look
    assert r.returncode == 1, "pins did not fail for %s (exit %d)\n%s" % (name, r.returncode, r.stdout[-1500:])
