"""The C-ABI library loads without a GPU, exports every symbol include/pz.h declares, and rejects
bad arguments on the host before anything is enqueued (no compute calls here)."""
import ctypes as C
import os
import re

import pytest

import paper_2602_11937_amd as pz
from paper_2602_11937_amd.binding import _CCache

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "pz.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pz_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"pz_kv_append_fp8", "pz_decode_attn", "pz_decode_attn_splitk_reduce"} <= set(names)
    lib = C.CDLL(pz.lib_path())
    for n in names:
        assert hasattr(lib, n), n


def test_host_side_helpers():
    assert pz.pz_decode_attn_n_splits(65536, 0, 1024) == 64
    assert pz.pz_decode_attn_n_splits(65536, 8192, 1024) == 9       # window + 63 positions at most
    assert pz.pz_decode_attn_n_splits(100, 8192, 1024) == 1
    assert pz.pz_decode_attn_n_splits(0, 0, 64) == 1
    assert pz.pz_decode_attn_n_splits(100, 0, 100) == 0             # not a multiple of 64
    assert pz.pz_decode_attn_workspace_bytes(16, 64, 64, 64) == 16 * 64 * 64 * 66 * 4
    assert pz.pz_decode_attn_workspace_bytes(0, 64, 64, 64) == 0
    assert pz.pz_status_string(0) == "PZ_OK" and "WORKSPACE" in pz.pz_status_string(-4)


def cache(**kw):
    a = dict(k=0x1000, v=0x2000, num_pages=4, page_size=64, n_kv_heads=8, head_dim=64, dtype=0)
    a.update(kw)
    return _CCache(a["k"], a["v"], a["num_pages"], a["page_size"], a["n_kv_heads"], a["head_dim"], a["dtype"])


def attn(c, **kw):
    a = dict(q=0x10, block_table=0x20, max_pages=4, seq_lens=0x30, batch=2, n_q_heads=64, sinks=None,
             sm_scale=0.125, k_scale=0.01, v_scale=0.01, window=0, split_tokens=0, n_splits=0, workspace=None,
             workspace_bytes=0, out=0x40, out_dtype=0)
    a.update(kw)
    return pz.pz_decode_attn(c, a["q"], a["block_table"], a["max_pages"], a["seq_lens"], a["batch"],
                             a["n_q_heads"], a["sinks"], a["sm_scale"], a["k_scale"], a["v_scale"], a["window"],
                             a["split_tokens"], a["n_splits"], a["workspace"], a["workspace_bytes"], a["out"],
                             a["out_dtype"], stream=0, check=False)


def test_decode_attn_rejects_bad_arguments_before_any_launch():
    NULL, SHAPE, UNSUP, WS = -1, -2, -3, -4
    assert attn(None) == NULL
    assert attn(cache(k=None)) == NULL
    assert attn(cache(), q=None) == NULL and attn(cache(), seq_lens=None) == NULL
    assert attn(cache(), out=None) == NULL
    assert attn(cache(head_dim=96)) == UNSUP and attn(cache(head_dim=256)) == UNSUP and attn(cache(page_size=48)) == UNSUP
    assert attn(cache(head_dim=128), batch=0) == 0                   # 128-channel heads are taken
    assert attn(cache(dtype=7)) == UNSUP
    assert attn(cache(), n_q_heads=60) == SHAPE                      # not a multiple of the KV heads
    assert attn(cache(n_kv_heads=1), n_q_heads=65) == UNSUP          # groups above 64
    assert attn(cache(n_kv_heads=1), n_q_heads=72) == UNSUP
    assert attn(cache(n_kv_heads=1), n_q_heads=128) == UNSUP
    for hq in (18, 22, 32, 34, 64, 48, 40, 128):                     # groups of 9, 11, 16, 17, 32, 24, 20, 64 are taken
        assert attn(cache(n_kv_heads=2), n_q_heads=hq, batch=0) == 0
    assert attn(cache(), batch=-1) == SHAPE and attn(cache(), window=-5) == SHAPE
    assert attn(cache(), sm_scale=0.0) == SHAPE and attn(cache(), k_scale=-1.0) == SHAPE
    assert attn(cache(), v_scale=float("nan")) == SHAPE
    assert attn(cache(), split_tokens=100) == UNSUP
    assert attn(cache(), split_tokens=128, n_splits=2) == WS
    assert attn(cache(), split_tokens=128, n_splits=2, workspace=0x50, workspace_bytes=100) == WS
    assert attn(cache(), split_tokens=128, n_splits=0, workspace=0x50, workspace_bytes=1 << 30) == SHAPE
    assert attn(cache(), out_dtype=3) == UNSUP
    # positions are 32-bit inside the kernels: a block-table row of more than 2^30 positions and
    # chunk grids that reach past 2^31 positions are refused
    assert attn(cache(page_size=64), max_pages=(1 << 24) + 1) == UNSUP
    assert attn(cache(page_size=16), max_pages=1 << 26, batch=0) == 0
    assert attn(cache(), split_tokens=1 << 20, n_splits=2048, workspace=0x50, workspace_bytes=1 << 40) == UNSUP
    assert attn(cache(), batch=0) == 0                               # nothing to do is not an error


def test_fused_append_call_validates_like_the_plain_call():
    NULL, SHAPE, UNSUP = -1, -2, -3

    def fused(c, k_new=0x50, v_new=0x60, **kw):
        a = dict(q=0x10, block_table=0x20, max_pages=4, seq_lens=0x30, batch=2, n_q_heads=64, sinks=None,
                 sm_scale=0.125, k_scale=0.01, v_scale=0.01, window=0, split_tokens=0, n_splits=0, workspace=None,
                 workspace_bytes=0, out=0x40, out_dtype=0)
        a.update(kw)
        return pz.pz_decode_attn_append(c, k_new, v_new, a["q"], a["block_table"], a["max_pages"], a["seq_lens"],
                                        a["batch"], a["n_q_heads"], a["sinks"], a["sm_scale"], a["k_scale"],
                                        a["v_scale"], a["window"], a["split_tokens"], a["n_splits"], a["workspace"],
                                        a["workspace_bytes"], a["out"], a["out_dtype"], stream=0, check=False)

    assert fused(cache(), k_new=None) == NULL and fused(cache(), v_new=None) == NULL
    assert fused(cache(), q=None) == NULL and fused(None) == NULL
    assert fused(cache(), n_q_heads=60) == SHAPE and fused(cache(head_dim=256)) == UNSUP
    assert fused(cache(), k_scale=0.0) == SHAPE
    assert fused(cache(), batch=0) == 0


def test_append_and_reduce_reject_bad_arguments():
    def app(c, **kw):
        a = dict(k_new=0x10, v_new=0x20, slots=0x30, n=4, ks=0.01, vs=0.01)
        a.update(kw)
        return pz.pz_kv_append_fp8(c, a["k_new"], a["v_new"], a["slots"], a["n"], a["ks"], a["vs"], stream=0,
                                   check=False)
    assert app(None) == -1 and app(cache(v=None)) == -1 and app(cache(), k_new=None) == -1
    assert app(cache(), slots=None) == -1
    assert app(cache(), n=-1) == -2 and app(cache(), ks=0.0) == -2
    assert app(cache(page_size=8)) == -3
    assert app(cache(), n=0) == 0

    def red(**kw):
        a = dict(ws=0x10, wsb=1 << 30, batch=2, hq=64, d=64, S=4, seq_lens=None, window=0, split=0, sinks=None,
                 vs=0.01, out=0x20, odt=0)
        a.update(kw)
        return pz.pz_decode_attn_splitk_reduce(a["ws"], a["wsb"], a["batch"], a["hq"], a["d"], a["S"],
                                               a["seq_lens"], a["window"], a["split"], a["sinks"], a["vs"],
                                               a["out"], a["odt"], stream=0, check=False)
    assert red(ws=None) == -4 and red(wsb=10) == -4
    assert red(out=None) == -1 and red(d=96) == -3 and red(d=128, batch=0) == 0 and red(S=0) == -2
    assert red(seq_lens=0x30, split=0) == -2 and red(vs=0.0) == -2
    assert red(seq_lens=0x30, split=(1 << 30) + 64) == -3
    assert red(batch=0) == 0


def test_error_wrapper_raises():
    with pytest.raises(pz.PzError) as e:
        pz.pz_decode_attn(cache(head_dim=96), 1, 1, 1, 1, 1, 8, None, 1, 1, 1, 0, 0, 0, None, 0, 1, stream=0)
    assert e.value.status == -3


def test_new_entry_points_reject_bad_arguments():
    lib = pz.lib()
    c = cache()
    # calibration
    assert pz.pz_kv_amax_update(None, 0x10, 8, 0x20, stream=0, check=False) == -1
    assert pz.pz_kv_amax_update(0x10, 0x20, -1, 0x30, stream=0, check=False) == -2
    assert pz.pz_kv_amax_update(0x11, 0x20, 8, 0x30, stream=0, check=False) == -3      # unaligned
    assert pz.pz_kv_amax_update(0x10, 0x20, 0, None, stream=0, check=False) == 0
    assert pz.pz_kv_scales_from_amax(None, 1, 0x10, stream=0, check=False) == -1
    # rotary + append
    def rope(cc, **kw):
        a = dict(q_in=0x10, q_out=0x10, k=0x20, v=0x30, pos=0x40, cos=0x50, sin=0x60, slots=0x70, n=4, hq=64, ks=0.01, vs=0.01)
        a.update(kw)
        return pz.pz_rope_kv_append_fp8(cc, a["q_in"], a["q_out"], a["k"], a["v"], a["pos"], a["cos"], a["sin"],
                                        a["slots"], a["n"], a["hq"], a["ks"], a["vs"], stream=0, check=False)
    assert rope(None) == -1 and rope(c, pos=None) == -1 and rope(c, cos=None) == -1 and rope(c, q_out=None) == -1
    assert rope(c, n=-1) == -2 and rope(c, ks=0.0) == -2 and rope(c, n=0) == 0
    assert rope(cache(head_dim=128)) == -3                                  # the rotary append is for 64-channel heads
    # prefill
    def pre(cc, **kw):
        a = dict(q=0x10, qs=0x20, bt=0x30, mp=4, sl=0x40, b=2, hq=64, mx=16, sinks=None, sm=0.125, ks=0.01, vs=0.01,
                 w=0, out=0x50, odt=0)
        a.update(kw)
        return pz.pz_prefill_attn(cc, a["q"], a["qs"], a["bt"], a["mp"], a["sl"], a["b"], a["hq"], a["mx"], a["sinks"],
                                  a["sm"], a["ks"], a["vs"], a["w"], a["out"], a["odt"], stream=0, check=False)
    assert pre(None) == -1 and pre(c, qs=None) == -1 and pre(c, out=None) == -1
    assert pre(c, hq=60) == -2 and pre(c, mx=-1) == -2 and pre(c, sm=0.0) == -2
    assert pre(cache(n_kv_heads=1), hq=65) == -3 and pre(c, odt=5) == -3    # a group of 65 heads
    assert pre(cache(head_dim=128)) == -3                                   # so is prefill
    assert pre(c, b=0) == 0 and pre(c, mx=0) == 0
    assert pre(cache(page_size=64), mp=(1 << 24) + 1) == -3                 # more than 2^30 positions per row
    # page pool
    assert lib.pz_page_pool_create(4, 16, 1, 0, 0) is None
    assert lib.pz_page_pool_append(None, 0) == -1 and lib.pz_page_pool_free_pages(None) == -1
    assert pz.pz_window_pages(-3, 16) == 0


def test_launch_override_entry_takes_only_its_listed_values():
    """pz_debug_set_launch_override: unknown overrides and values outside the listed ones are refused; a
    negative value (and 0 for the two counts) hands the choice back.  No environment variable is read by
    the library: the names the earlier test knobs had do not occur in it."""
    f = pz.lib().pz_debug_set_launch_override
    assert f(-1, 1) == -2 and f(5, 1) == -2
    for which in (2, 3, 4):
        assert f(which, 2) == -2
        assert f(which, 0) == 0 and f(which, 1) == 0 and f(which, -1) == 0
    for which in (0, 1):
        assert f(which, 8) == 0 and f(which, 0) == 0 and f(which, -5) == 0
    assert pz.pz_debug_set_launch_override("attn_waves", -1) == 0
    blob = open(pz.lib_path(), "rb").read()
    for name in (b"PZ_ATTN_WAVES", b"PZ_APPEND_FORM", b"PZ_APPEND_FUSED", b"PZ_ATTN_BALANCED", b"getenv"):
        assert name not in blob, name


def test_header_is_plain_c_and_a_c_program_links_against_the_library(tmp_path):
    """include/pz.h compiles as C99 with nothing but <stddef.h> / <stdint.h>, and a C program that calls the
    host-side entry points links against libpz.so and gets the documented values (no GPU involved)."""
    import subprocess
    src = tmp_path / "use_pz.c"
    src.write_text(r'''
#include "pz.h"
#include <stdio.h>
int main(void) {
    pz_cache c = {0};
    if (pz_decode_attn_n_splits(65536, 0, 1024) != 64) return 1;
    if (pz_decode_attn_workspace_bytes(16, 64, 64, 64) != (size_t)16 * 64 * 64 * 66 * 4) return 2;
    if (pz_window_pages(8192, 64) != 129) return 3;
    if (pz_kv_append_fp8(&c, 0, 0, 0, 1, 1.0f, 1.0f, 0) != PZ_ERR_NULL) return 4;       /* refused on the host */
    if (pz_decode_attn_noalloc(0, 0, 0, 1, 0, 1, 8, 0, 1.f, 1.f, 1.f, 0, 64, 1, (void *)8, PZ_OUT_F32, 0) != PZ_ERR_NULL) return 5;
    if (pz_debug_set_launch_override(PZ_OVERRIDE_COUNT, 1) != PZ_ERR_SHAPE) return 6;
    if (PZ_NOALLOC_WORKSPACE_BYTES != (32u << 20)) return 7;
    printf("%s\n", pz_status_string(PZ_ERR_WORKSPACE));
    return 0;
}
''')
    exe = tmp_path / "use_pz"
    lib_dir = os.path.dirname(pz.lib_path())
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), str(src),
                        "-o", str(exe), "-L", lib_dir, "-l:libpz.so", "-Wl,-rpath," + lib_dir],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0 and "WORKSPACE" in r.stdout, (r.returncode, r.stdout, r.stderr)


def test_bench_reports_counter_traffic_only_for_the_sources_it_was_measured_on(tmp_path, monkeypatch):
    import bench
    kernel = "decode_attn_balanced_kernel<64,1>"
    got, why = bench.traffic_from_profile("cfg3", kernel)
    line = [l for l in open(os.path.join(ROOT, "profiles", "decode_step_cfg3_fp8_hbm_traffic.txt")) if l.startswith("bench.py reads:")]
    assert len(line) == 1
    recorded = re.search(r"source_sha256=([0-9a-f]+)", line[0]).group(1)
    if recorded == bench.kernel_source_hash():
        assert got == int(re.search(r"traffic_bytes_per_launch=(\d+)", line[0]).group(1)) and "profiles/" in why
    else:
        assert got is None and "measure again" in why
    monkeypatch.setattr(bench, "kernel_source_hash", lambda: "0" * 16)
    got, why = bench.traffic_from_profile("cfg3", kernel)
    assert got is None and "measure again" in why
    assert bench.traffic_from_profile("cfg4_w128", kernel)[0] is None
