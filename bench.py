#!/usr/bin/env python3
"""Benchmark of the decode-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one pass of the whole path over one batch: quantise-and-append of one new token per
sequence, decode attention (split-K partials + log-sum-exp merge, or single pass for short
windows), all through the C ABI (paper_2602_11937_amd.decode_step issues the calls).  Inputs are
seeded synthetic gpt-oss-shaped tensors, resident in HBM before the timed region.  Consecutive steps
walk over several independent cache instances so that no step re-reads data the 256 MB Infinity
Cache may still hold.

Prints ONE JSON line.  Without --workload it is the headline configuration (cfg3: batch 16 x context
65536, FP8 KV): metric / value (algorithmic GB/s of the whole step) / ms_per_step, `roofline` (the
dominant kernel: algorithmic bytes per launch over its event-timed duration, against the 8 TB/s HBM
peak, plus the HBM traffic measured with hardware counters when the committed counter summary was
taken from the very kernel sources that are running), `cpu_baseline` (the CPU oracle timed on the
same workload, with a parity figure), `bf16_kv`, `repetitions`, `fused_append`, `stream_read`,
`hip_graph`, `tuned_split`, and `all_configs`: the other benchmark configurations (cfg2, cfg4 at
window 128 and 8192, the 36-layer cfg5 step) and the widened rows (max calibration, prefill, the
window page pool, the fused rotary append, 128-channel heads), each run through the same code as `--workload NAME` with
fewer repetitions and reported as step time, kernel fraction of its roofline and oracle parity.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

METRIC = "decode-attention GB/s (% of HBM peak) + attn tokens/s, B=16 ctx=64K FP8 KV"
HBM_PEAK_GBPS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
DTYPE = "e4m3 KV -> bf16 MFMA operands, f32 accumulate"
CFG5_SPLIT = 8192      # split-K chunk length of cfg5's full and window-8192 layers (the configuration names none).
                       # Per step at 1024 / 2048 / 4096 / 8192 / 16384: a full layer 314.4 / 312.8 / 312.8 / 311.3 /
                       # 386.2 us, a window-8192 layer 50.9 / 51.4 / 50.9 / 50.1 / 49.1 us

WORKLOADS = {
    # name: (B, seq_lens spec, window, split_tokens, outlier_frac, seed, instances, description)
    "cfg3": dict(B=16, L=65536, window=0, split_tokens=1024, outlier_frac=0.01, seed=3, instances=4,
                 text="cfg3: batch 16 x context 65536, 64 q / 8 KV heads, d=64, paged E4M3 KV (page 64, random "
                      "page table), 1% outlier K channels x20, sinks; kv_append of 1 token/seq + split-K "
                      "(1024-token chunks) decode attention + LSE merge"),
    "cfg2": dict(B=64, L=8192, window=0, split_tokens=1024, outlier_frac=0.0, seed=2, instances=6,
                 text="cfg2: batch 64 x context 8192, 64 q / 8 KV heads, d=64, paged E4M3 KV (page 64); "
                      "kv_append + split-K (1024) decode attention + LSE merge"),
    "cfg4_w128": dict(B=256, L=(1024, 65536), window=128, split_tokens=0, outlier_frac=0.0, seed=4, instances=2,
                      text="cfg4: batch 256, ragged contexts U[1024,65536], sliding window 128, single pass"),
    "cfg4_w8192": dict(B=256, L=(1024, 65536), window=8192, split_tokens=1024, outlier_frac=0.0, seed=4,
                       instances=2,
                       text="cfg4: batch 256, ragged contexts U[1024,65536], sliding window 8192, split-K 1024"),
    # diagnostics: uniform lengths at twice cfg3's batch, and cfg3's batch with ragged lengths
    "diag_b32_uniform": dict(B=32, L=65536, window=0, split_tokens=1024, outlier_frac=0.0, seed=7, instances=3,
                             text="diagnostic: batch 32 x context 65536, split-K 1024"),
    "diag_b40_uniform": dict(B=40, L=65536, window=0, split_tokens=1024, outlier_frac=0.0, seed=9, instances=2,
                             text="diagnostic: batch 40 x context 65536, split-K 1024 (20 chunks per SIMD-wave)"),
    "diag_b8_128k": dict(B=8, L=131072, window=0, split_tokens=1024, outlier_frac=0.0, seed=8, instances=4,
                         text="diagnostic: batch 8 x context 131072, split-K 1024"),
    "diag_b16_ragged": dict(B=16, L=(1024, 131072), window=0, split_tokens=1024, outlier_frac=0.0, seed=5, instances=4,
                            text="diagnostic: batch 16, ragged contexts U[1024,131072], split-K 1024"),
    # what one GPU of a tensor-parallel group of 8 holds of cfg3: one KV head and its 8 query heads
    "diag_tp8_shard": dict(B=16, L=65536, window=0, split_tokens=1024, outlier_frac=0.01, seed=3, instances=8, Hq=8, Hkv=1,
                           text="diagnostic: cfg3 sharded over KV heads for tensor parallelism 8 (1 KV head + 8 query heads "
                                "per GPU): batch 16 x context 65536, split-K 1024"),
    # 128-channel heads (not the paper's model: the boundary's second head dimension), as many KV bytes as cfg3
    "diag_d128": dict(B=16, L=32768, window=0, split_tokens=1024, outlier_frac=0.0, seed=11, instances=4, d=128,
                      text="diagnostic: head dimension 128: batch 16 x context 32768, 64 q / 8 KV heads, split-K 1024"),
    # single layers of the heterogeneous step (cfg5), for tests and tuning
    "cfg5_full": dict(B=32, L=(1024, 131072), window=0, split_tokens=CFG5_SPLIT, outlier_frac=0.0, seed=5, instances=3,
                      bounded=True, text="cfg5 full-attention layer: batch 32, ragged contexts U[1024,131072], split-K %d" % CFG5_SPLIT),
    "cfg5_w8192": dict(B=32, L=(1024, 131072), window=8192, split_tokens=CFG5_SPLIT, outlier_frac=0.0, seed=5, instances=3,
                       bounded=True, text="cfg5 window-8192 layer: batch 32, ragged contexts U[1024,131072], split-K %d" % CFG5_SPLIT),
    "cfg5_w128": dict(B=32, L=(1024, 131072), window=128, split_tokens=0, outlier_frac=0.0, seed=5, instances=3,
                      bounded=True, text="cfg5 window-128 layer: batch 32, ragged contexts U[1024,131072], single pass"),
}
OTHER_WORKLOADS = ["cfg5", "calib", "prefill", "pool", "rope"]
# what the default run reports besides the headline, in this order
ALL_CONFIGS = ["cfg2", "cfg4_w128", "cfg4_w8192", "cfg5", "calib", "prefill", "pool", "rope", "diag_d128"]

# Sources that decide what the decode-attention launches do.  The HBM-traffic figure in profiles/ was
# measured with hardware counters on a build of exactly these bytes; the summary records their hash.
KERNEL_SOURCES = ["pz_api.hip", "pz_attn.hip", "pz_attn_balanced.hip", "pz_attn_common.h", "pz_attn_steps.h",
                  "pz_internal.h", "pz_quant.h"]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kernel_source_hash() -> str:
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2602_11937_amd", "csrc", name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read() + b"\0")
    return h.hexdigest()[:16]


def traffic_from_profile(workload: str, kernel: str):
    """HBM bytes per launch of `kernel` on `workload` from the committed counter summary
    (profiles/decode_step_<workload>_fp8_hbm_traffic.txt), or (None, why) when there is no summary or it
    was taken from other kernel sources than the ones that are running."""
    path = os.path.join(ROOT, "profiles", "decode_step_%s_fp8_hbm_traffic.txt" % workload)
    if not os.path.exists(path):
        return None, "no counter summary for this workload under profiles/"
    want = kernel_source_hash()
    for line in open(path):
        m = re.match(r"bench\.py reads: kernel=(\S+) traffic_bytes_per_launch=(\d+) source_sha256=([0-9a-f]+)", line.strip())
        if m and m.group(1) == kernel:
            if m.group(3) != want:
                return None, ("the counter summary %s was taken from kernel sources %s, this build is %s: measure again"
                              % (os.path.basename(path), m.group(3), want))
            return int(m.group(2)), "rocprofv3 FETCH_SIZE + WRITE_SIZE per launch, from profiles/%s" % os.path.basename(path)
    return None, "the counter summary has no line for " + kernel


def host_cores() -> int:
    """Threads the oracle is given: every core this process may run on, held to the CPU share the machine
    states for a job (its OMP_NUM_THREADS setting) where it states one: a GPU machine hands each job a share of
    a larger host."""
    n = len(os.sched_getaffinity(0))
    share = os.environ.get("OMP_NUM_THREADS", "")
    return max(1, min(n, int(share))) if share.isdigit() and int(share) > 0 else n


# ------------------------------------------------------------------ one layer = one cache instance

class Layer:
    """One cache instance + everything a step on it needs, with the C-ABI arguments prepared."""

    def __init__(self, pz, wl, torch, spec, seed, kv_dtype, keep_context=False):
        from paper_2602_11937_amd.decode_step import DecodeLayer
        B = spec["B"]
        if isinstance(spec["L"], tuple):
            seq_lens = wl.ragged_lengths(spec["seed"], B, *spec["L"])
        else:
            seq_lens = np.full(B, spec["L"], dtype=np.int32)
        self.pz, self.torch = pz, torch
        self.window, self.split = spec["window"], spec["split_tokens"]
        self.kv_dtype = kv_dtype
        # a window layer keeps only the pages its window can touch (spec["bounded"])
        resident = self.window + 64 if (spec.get("bounded") and self.window > 0) else None
        lay = wl.device_layer(B=B, Hq=spec.get("Hq", 64), Hkv=spec.get("Hkv", 8), d=spec.get("d", 64), seq_lens=seq_lens,
                              window=self.window,
                              seed=seed, outlier_frac=spec["outlier_frac"], resident=resident)
        self.lay = lay
        self.k_scale = lay.k_scale if kv_dtype == pz.KV_FP8 else 1.0
        self.v_scale = lay.v_scale if kv_dtype == pz.KV_FP8 else 1.0
        self.cache = pz.PagedCache.allocate(lay.num_pages, lay.P, lay.Hkv, lay.d, kv_dtype, "cuda")
        slots = torch.from_numpy(lay.slot_mapping_host).to("cuda")
        T = slots.numel()
        step = 1 << 20
        for t0 in range(0, T, step):
            n = min(step, T - t0)
            pz.pz_kv_append_fp8(self.cache, lay.k_ctx[t0:t0 + n], lay.v_ctx[t0:t0 + n], slots[t0:t0 + n], n,
                                self.k_scale, self.v_scale)
        torch.cuda.synchronize()
        if not keep_context:
            lay.k_ctx = lay.v_ctx = None
        del slots
        self.out = torch.empty((B, lay.Hq, lay.d), dtype=torch.float32, device="cuda")
        self.max_pages = int(lay.block_table_host.shape[1])
        self.dl = DecodeLayer(cache=self.cache, block_table=lay.block_table, max_pages=self.max_pages,
                              window=self.window, k_scale=self.k_scale, v_scale=self.v_scale, sm_scale=lay.sm_scale,
                              sinks=lay.sinks, split_tokens=self.split)
        self.set_split(self.split)

    def set_split(self, split_tokens, workspace=None):
        """(Re)size the split-K workspace for a chunk length (0 = single pass); `workspace` shares one."""
        lay = self.lay
        self.split = self.dl.split_tokens = split_tokens
        max_len = int(lay.seq_lens.max())
        self.S = self.dl.n_splits(max_len)
        self.ws_bytes = self.dl.workspace_bytes(lay.B, lay.Hq, max_len)
        self.ws = workspace if workspace is not None else \
            self.torch.empty((max(self.ws_bytes, 4) // 4,), dtype=self.torch.float32, device="cuda")

    # algorithmic bytes: what the method must move (split-K workspace traffic is overhead)
    def attn_bytes(self, wl):
        lay = self.lay
        eb = 1 if self.kv_dtype == self.pz.KV_FP8 else 2
        toks = wl.kv_tokens_read(lay.seq_lens, self.window)
        L = lay.seq_lens.astype(np.int64)
        span = np.minimum(L, self.window) if self.window > 0 else L
        bt_entries = int(((span + lay.P - 1) // lay.P + 1).sum())
        return toks * wl.kv_bytes_per_token(lay.Hkv, lay.d, eb) + lay.B * lay.Hq * lay.d * 2 + bt_entries * 4 \
            + lay.B * 4

    def step_bytes(self, wl):
        lay = self.lay
        eb = 1 if self.kv_dtype == self.pz.KV_FP8 else 2
        append = lay.B * lay.Hkv * lay.d * 2 * (2 + eb) + lay.B * 8
        final = lay.B * lay.Hq * lay.d * 4 + lay.Hq * 4
        return self.attn_bytes(wl) + append + final

    def append(self):
        lay = self.lay
        self.dl.append(lay.k_new, lay.v_new, lay.new_slots, lay.B)

    def attn(self):
        lay = self.lay
        self.dl.attend(lay.q, lay.seq_lens_dev, lay.B, lay.Hq, self.S, self.ws, self.ws_bytes, self.out)

    def reduce(self):
        lay = self.lay
        self.dl.merge(lay.seq_lens_dev, lay.B, lay.Hq, self.S, self.ws, self.ws_bytes, self.out)

    def step_fused(self):
        """pz_decode_attn_append (+ merge): the append of the step's new token inside the attention call."""
        lay = self.lay
        self.dl.step(lay.q, lay.k_new, lay.v_new, lay.new_slots, lay.seq_lens_dev, lay.B, lay.Hq, self.S, self.ws,
                     self.ws_bytes, self.out, fused=True)

    def step(self, ev=None):
        if ev is None:
            lay = self.lay
            self.dl.step(lay.q, lay.k_new, lay.v_new, lay.new_slots, lay.seq_lens_dev, lay.B, lay.Hq, self.S, self.ws,
                         self.ws_bytes, self.out)
            return
        self.append()
        ev[0].record()
        self.attn()
        ev[1].record()
        self.reduce()


def time_fused(torch, layers, steps, warmup):
    """The same K steps with two launches each: pz_decode_attn_append + merge."""
    for i in range(warmup):
        layers[i % len(layers)].step_fused()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        layers[(warmup + i) % len(layers)].step_fused()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def time_steps(torch, layers, steps, warmup, events):
    """W untimed steps, then exactly K timed steps between synchronisations.  With events=True the
    dominant kernel (decode attention) is bracketed by events on the launch stream in every timed
    step; the two event records cost about 5 us per step, so the step time that is reported as
    `value` comes from a pass without them."""
    for i in range(warmup):
        layers[i % len(layers)].step()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        layers[(warmup + i) % len(layers)].step(evs[i] if events else None)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kern_ms = np.array([a.elapsed_time(b) for a, b in evs]) if events else None
    return (t1 - t0) * 1e3 / steps, kern_ms


def capture(torch, fn):
    """Record fn's launches (kernels only: the library enqueues nothing else) into a HIP graph."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    return graph


def time_graphs(torch, graphs, steps, warmup):
    """The same K timed steps, each step one replay of a pre-recorded HIP graph."""
    for i in range(warmup):
        graphs[i % len(graphs)].replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        graphs[(warmup + i) % len(graphs)].replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def oracle_sample(oracle, torch, layer, seqs):
    """Oracle-side copy of the listed sequences of a Layer: its own cache (compact page numbering,
    its own layout) filled by the oracle's quantise-and-append from the same bf16 K/V, all but the
    newest token of each sequence.  Returns (kc, vc, block_table, q_bits, new_k, new_v, new_slots)."""
    lay = layer.lay
    P = lay.P
    off, fp0 = lay.ctx_offsets, lay.first_pos
    # a window layer never attends to positions before its window: the oracle's copy starts at the page that
    # holds the window's first position (the entries before it stay -1)
    fp = np.array(fp0, dtype=np.int64)
    if layer.window > 0:
        L64 = lay.seq_lens.astype(np.int64)
        fp = np.maximum(fp, (np.maximum(L64 - layer.window, 0) // P) * P)
    end_page = [-(-int(lay.seq_lens[b]) // P) for b in seqs]
    bt = np.full((len(seqs), max(end_page)), -1, dtype=np.int32)
    at = 0
    for i, b in enumerate(seqs):
        p0 = int(fp[b]) // P
        bt[i, p0:end_page[i]] = np.arange(at, at + end_page[i] - p0)
        at += end_page[i] - p0
    kc, vc = oracle.new_cache(at * P, lay.Hkv, lay.d, oracle.KV_FP8)
    new_k, new_v, new_slots = [], [], []
    for i, b in enumerate(seqs):
        skip = int(fp[b] - fp0[b])                  # resident rows of the sequence that lie before the window
        kb = lay.k_ctx[off[b] + skip:off[b + 1]].view(torch.int16).cpu().numpy().view(np.uint16)
        vb = lay.v_ctx[off[b] + skip:off[b + 1]].view(torch.int16).cpu().numpy().view(np.uint16)
        j = np.arange(int(fp[b]), int(lay.seq_lens[b]), dtype=np.int64)
        slots = bt[i, j // P].astype(np.int64) * P + j % P
        oracle.kv_append(kc, vc, kb[:-1], vb[:-1], slots[:-1], lay.k_scale, lay.v_scale)
        new_k.append(kb[-1:]); new_v.append(vb[-1:]); new_slots.append(slots[-1:])
    q = lay.q[torch.as_tensor(list(seqs), device=lay.q.device)].view(torch.int16).cpu().numpy().view(np.uint16)
    return kc, vc, bt, q, np.concatenate(new_k), np.concatenate(new_v), np.concatenate(new_slots)


def cpu_baseline(pz, wl, oracle, torch, layer, n_seq):
    """The oracle, as it stands, on the first n_seq sequences of a Layer (all query heads), on every
    host core this process may use: its own quantise-and-append of their context (set-up, untimed),
    then timed: append of the new tokens + unsplit attention.  Returns the baseline dict and the
    oracle rows (fp32 pass, fp64 pass)."""
    lay = layer.lay
    cores = host_cores()
    seqs = list(range(n_seq))
    kc, vc, bt, q, new_k, new_v, new_slots = oracle_sample(oracle, torch, layer, seqs)
    sinks = lay.sinks.cpu().numpy()
    t0 = time.perf_counter()
    oracle.kv_append(kc, vc, new_k, new_v, new_slots, lay.k_scale, lay.v_scale)
    want = oracle.decode_attn(kc, vc, lay.P, q, bt, lay.seq_lens[:n_seq], sinks, lay.sm_scale, lay.k_scale,
                              lay.v_scale, layer.window, nthreads=cores)
    dt = time.perf_counter() - t0
    # untimed: the same rows with fp64 accumulation, the reference of the parity figure (the fp32 pass sums up to
    # 65536 terms one after the other and is itself up to L * 2^-24 away from it)
    want64 = oracle.decode_attn(kc, vc, lay.P, q, bt, lay.seq_lens[:n_seq], sinks, lay.sm_scale, lay.k_scale,
                                lay.v_scale, layer.window, accum="f64", nthreads=cores)
    toks = wl.kv_tokens_read(lay.seq_lens[:n_seq], layer.window)
    nbytes = toks * wl.kv_bytes_per_token(lay.Hkv, lay.d, 1)
    base = {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
            "seconds": dt, "attn_tokens_per_s": n_seq / dt, "timed": "the oracle's fp32 pass",
            "sample": "%s %d of %d sequences of cache instance 0, all %d query heads: oracle kv_append of "
                      "their new tokens + unsplit fp32 decode attention (%d cached tokens)"
                      % ("all" if n_seq == lay.B else "first", n_seq, lay.B, lay.Hq, toks)}
    return base, want, want64


# ------------------------------------------------------------------ single-layer workloads (cfg2, cfg3, cfg4, diagnostics)

def run_layer_workload(args, pz, wl, torch, name, light=False):
    spec = dict(WORKLOADS[name])
    if args.split_tokens is not None and not light:
        spec["split_tokens"] = args.split_tokens
        spec["text"] += " [split_tokens overridden to %d]" % args.split_tokens
    steps, warmup = (min(args.steps, 100), min(args.warmup, 50)) if light else (args.steps, args.warmup)
    # the oracle's sample: the whole batch on the headline run (about 5 s of CPU work on 16 cores), a few
    # sequences of the large batches
    if args.cpu_seqs is not None:
        cpu_seqs = args.cpu_seqs
    else:
        whole = name in ("cfg3", "cfg2", "cfg4_w128") or (name == "cfg4_w8192" and not light)
        cpu_seqs = spec["B"] if whole else min(spec["B"], 32 if name == "cfg4_w8192" else 8)
    if args.calib_copy:
        src = torch.ones((768 << 20) // 4, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    t_setup = time.perf_counter()
    layers = [Layer(pz, wl, torch, spec, seed=spec["seed"] + 1000 * r, kv_dtype=pz.KV_FP8,
                    keep_context=(r == 0 and cpu_seqs > 0)) for r in range(spec["instances"])]
    log("%s: built %d FP8 cache instances in %.1f s" % (name, len(layers), time.perf_counter() - t_setup))
    ms_step, _ = time_steps(torch, layers, steps, warmup, events=False)
    # three more timed regions of the same K steps: spread of the step time between repetitions
    reps = [ms_step] + [time_steps(torch, layers, steps, 2, events=False)[0] for _ in range(1 if light else 3)]
    ms_step_ev, kern_ms = time_steps(torch, layers, steps, warmup, events=True)
    attn_bytes = float(np.mean([l.attn_bytes(wl) for l in layers]))
    step_bytes = float(np.mean([l.step_bytes(wl) for l in layers]))
    B = spec["B"]
    kern_avg_ms = float(kern_ms.mean())
    kernel = "decode_attn_balanced_kernel<64,1>" if spec["window"] == 0 and spec["split_tokens"] > 0 \
        else "decode_attn_kernel<64,1>"
    if spec.get("d", 64) == 128:
        kernel = "decode_attn_d128_kernel<64,1>"
    traffic, traffic_note = (None, "split_tokens overridden") if (args.split_tokens is not None and not light) \
        else traffic_from_profile(name, kernel)
    result = {
        "metric": METRIC if name == "cfg3" else METRIC.split(", B=16")[0] + ", " + name + " FP8 KV",
        "value": step_bytes / (ms_step * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": ms_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": spec["text"], "batch": B, "n_q_heads": spec.get("Hq", 64), "n_kv_heads": spec.get("Hkv", 8), "head_dim": 64,
                   "page_size": 64, "window": spec["window"], "split_tokens": spec["split_tokens"],
                   "cache_instances_rotated": len(layers)},
        "attn_tokens_per_s": B / (ms_step * 1e-3),
        "pct_hbm_peak": 100.0 * step_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "repetitions": {"n": len(reps), "ms_per_step_mean": float(np.mean(reps)), "ms_per_step_std": float(np.std(reps))},
        "roofline": {"bound": "hbm", "kernel": kernel,
                     "achieved": attn_bytes / (kern_avg_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": attn_bytes / (kern_avg_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "kernel_us_avg": kern_avg_ms * 1e3, "kernel_us_std": float(kern_ms.std() * 1e3),
                     "ms_per_step_with_events": ms_step_ev,
                     "algorithmic_bytes_per_launch": attn_bytes,
                     "traffic": traffic, "traffic_source": traffic_note},
    }
    ms_f = time_fused(torch, layers, steps, warmup)
    result["fused_append"] = {"ms_per_step": ms_f, "GBps": step_bytes / (ms_f * 1e-3) / 1e9,
                              "pct_hbm_peak": 100.0 * step_bytes / (ms_f * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                              "attn_tokens_per_s": B / (ms_f * 1e-3),
                              "launches": "pz_decode_attn_append + pz_decode_attn_splitk_reduce"
                              if spec["split_tokens"] else "pz_decode_attn_append"}
    # the box's plain streaming-read rate over the very same cache bytes: the library's amax kernel
    # (16-byte loads, a max per element, nothing written) run over the K and V arrays of each instance
    if name in ("cfg3", "cfg2") and not light:
        amax = torch.zeros(2, dtype=torch.float32, device="cuda")
        n_el = layers[0].cache.k.numel() // 2
        for l in layers:
            pz.pz_kv_amax_update(l.cache.k, l.cache.v, n_el, amax)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
        for i, (a, b) in enumerate(evs):
            l = layers[i % len(layers)]
            a.record()
            pz.pz_kv_amax_update(l.cache.k, l.cache.v, n_el, amax)
            b.record()
        torch.cuda.synchronize()
        ms_r = float(np.mean([a.elapsed_time(b) for a, b in evs]))
        rd = 2.0 * layers[0].cache.k.numel() / (ms_r * 1e-3) / 1e9
        result["stream_read"] = {"GBps": rd, "pct_hbm_peak": 100.0 * rd / HBM_PEAK_GBPS, "kernel": "kv_amax_kernel over "
                                 "the K and V arrays of the same cache instances (sequential addresses)",
                                 "attn_kernel_pct_of_it": 100.0 * result["roofline"]["achieved"] / rd}
    if not light:
        # the same step launched as one replay of a recorded HIP graph (one graph per cache instance)
        graphs = [capture(torch, l.step) for l in layers]
        ms_g = time_graphs(torch, graphs, steps, warmup)
        result["hip_graph"] = {"ms_per_step": ms_g, "GBps": step_bytes / (ms_g * 1e-3) / 1e9,
                               "pct_hbm_peak": 100.0 * step_bytes / (ms_g * 1e-3) / 1e9 / HBM_PEAK_GBPS}
        del graphs
    if name == "cfg3" and args.split_tokens is None and not light:
        # the same step with the chunk length a caller free to choose would use (fewer, longer partials)
        for l in layers:
            l.set_split(8192)
        ms_t, _ = time_steps(torch, layers, steps, warmup, events=False)
        result["tuned_split"] = {"split_tokens": 8192, "ms_per_step": ms_t, "GBps": step_bytes / (ms_t * 1e-3) / 1e9,
                                 "pct_hbm_peak": 100.0 * step_bytes / (ms_t * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                                 "attn_tokens_per_s": B / (ms_t * 1e-3)}
        for l in layers:
            l.set_split(spec["split_tokens"])

    if cpu_seqs > 0:
        import oracle
        n_seq = min(cpu_seqs, B)
        layers[0].out.fill_(float("nan"))
        layers[0].step()
        torch.cuda.synchronize()
        got = layers[0].out[:n_seq].cpu().numpy()
        base, want, want64 = cpu_baseline(pz, wl, oracle, torch, layers[0], n_seq)
        rms = float(np.sqrt(np.mean(want64.astype(np.float64) ** 2)))
        base["parity_max_abs_over_rms"] = float(np.max(np.abs(got - want64)) / rms)
        base["parity_vs_fp32_pass"] = float(np.max(np.abs(got - want)) / rms)
        log("%s: oracle on %d sequences: %.1f s on %d cores, parity %.2e of output RMS"
            % (name, n_seq, base["seconds"], base["cores"], base["parity_max_abs_over_rms"]))
        result["cpu_baseline"] = base
        layers[0].lay.k_ctx = layers[0].lay.v_ctx = None
    else:
        result["cpu_baseline"] = None

    if not args.no_bf16 and not light:
        del layers
        torch.cuda.empty_cache()
        n_inst = max(2, spec["instances"] - 1)
        bl = [Layer(pz, wl, torch, spec, seed=spec["seed"] + 1000 * r, kv_dtype=pz.KV_BF16) for r in range(n_inst)]
        ms_b, _ = time_steps(torch, bl, steps, warmup, events=False)
        _, kern_b = time_steps(torch, bl, steps, warmup, events=True)
        sb = float(np.mean([l.step_bytes(wl) for l in bl]))
        ab = float(np.mean([l.attn_bytes(wl) for l in bl]))
        result["bf16_kv"] = {"ms_per_step": ms_b, "GBps": sb / (ms_b * 1e-3) / 1e9,
                             "attn_tokens_per_s": B / (ms_b * 1e-3), "kernel_us_avg": float(kern_b.mean() * 1e3),
                             "kernel_GBps": ab / (float(kern_b.mean()) * 1e-3) / 1e9,
                             "fp8_speedup_tokens_per_s": ms_b / ms_step}
    return result


# ------------------------------------------------------------------ cfg5: the heterogeneous 36-layer step

class Model:
    """The heterogeneous 36-layer decode step: every layer appends one token per sequence and runs its
    attention (window 128: single pass; window 8192 and full: split-K with `split_tokens`-long chunks + merge).
    All layers write their split-K partials to ONE workspace, as a serving loop would."""

    def __init__(self, pz, wl, torch, kv_dtype, keep_context_types=(), split_tokens=1024):
        self.pattern = wl.layer_pattern(seed=5)
        self.layers = []
        kept = set()
        for i, w in enumerate(self.pattern):
            spec = dict(B=32, L=(1024, 131072), window=w, split_tokens=0 if w == 128 else split_tokens,
                        outlier_frac=0.0, seed=5, bounded=True)
            keep = w in keep_context_types and w not in kept
            kept.add(w) if keep else None
            self.layers.append(Layer(pz, wl, torch, spec, seed=5 + 1000 * (i + 1), kv_dtype=kv_dtype,
                                     keep_context=keep))
        shared = max(self.layers, key=lambda l: l.ws_bytes).ws
        for l in self.layers:
            l.set_split(l.split, workspace=shared)
        self.full = [l for l in self.layers if l.window == 0]

    def step(self, ev=None):
        k = 0
        for l in self.layers:
            if ev is not None and l.window == 0:
                l.step(ev[k])
                k += 1
            else:
                l.step()


def time_model_fused(torch, model, steps, warmup):
    for _ in range(warmup):
        for l in model.layers:
            l.step_fused()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        for l in model.layers:
            l.step_fused()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def time_model(torch, model, steps, warmup, events):
    for _ in range(warmup):
        model.step()
    n_full = len(model.full)
    evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_full)]
           for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        model.step(evs[i] if events else None)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kern = np.array([[a.elapsed_time(b) for a, b in e] for e in evs]) if events else None
    return (t1 - t0) * 1e3 / steps, kern


def run_cfg5(args, pz, wl, torch, light=False):
    """36 layers: 18 x window 128, 8 x window 8192, 10 x full; batch 32, contexts U[1024,131072]."""
    split5 = args.split_tokens if (args.split_tokens is not None and not light) else CFG5_SPLIT
    steps, warmup = (min(args.steps, 20), min(args.warmup, 5)) if light else (min(args.steps, 50), min(args.warmup, 10))
    cpu_seqs = args.cpu_seqs if args.cpu_seqs is not None else 2
    text = ("cfg5: 36-layer decode step (18 x window-128, 8 x window-8192, 10 x full attention), batch 32, ragged "
            "contexts U[1024,131072], 64 q / 8 KV heads, d=64, paged E4M3 KV with per-layer K/V scales; every layer "
            "= kv_append of 1 token/seq + decode attention (+ LSE merge; split-K chunks of %d tokens)" % split5)
    t0 = time.perf_counter()
    model = Model(pz, wl, torch, pz.KV_FP8, keep_context_types=(128, 8192, 0) if cpu_seqs > 0 else (),
                  split_tokens=split5)
    log("cfg5: built the 36 FP8 layer caches in %.1f s" % (time.perf_counter() - t0))
    ms_step, _ = time_model(torch, model, steps, warmup, events=False)
    reps = [ms_step] + [time_model(torch, model, steps, 1, events=False)[0] for _ in range(1 if light else 3)]
    ms_ev, kern = time_model(torch, model, steps, warmup, events=True)
    step_bytes = float(sum(l.step_bytes(wl) for l in model.layers))
    full_bytes = float(np.mean([l.attn_bytes(wl) for l in model.full]))
    kern_avg = float(kern.mean())
    B = 32
    by_type = {}
    for w in (128, 8192, 0):
        ls = [l for l in model.layers if l.window == w]
        by_type["full" if w == 0 else "window_%d" % w] = {"layers": len(ls),
                                                             "kv_bytes_per_layer": float(ls[0].attn_bytes(wl))}
    result = {
        "metric": "decode-attention GB/s (% of HBM peak) + attn tokens/s, 36-layer heterogeneous step B=32 FP8 KV",
        "value": step_bytes / (ms_step * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": text, "batch": B, "layers": by_type},
        "attn_tokens_per_s": B / (ms_step * 1e-3),
        "pct_hbm_peak": 100.0 * step_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "repetitions": {"n": len(reps), "ms_per_step_mean": float(np.mean(reps)), "ms_per_step_std": float(np.std(reps))},
        "roofline": {"bound": "hbm", "kernel": "decode_attn_balanced_kernel<64,1> (the 10 full-attention layers)",
                     "achieved": full_bytes / (kern_avg * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": full_bytes / (kern_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS, "kernel_us_avg": kern_avg * 1e3,
                     "ms_per_step_with_events": ms_ev, "algorithmic_bytes_per_launch": full_bytes, "traffic": None},
    }
    ms_f = time_model_fused(torch, model, steps, warmup)
    result["fused_append"] = {"ms_per_step": ms_f, "GBps": step_bytes / (ms_f * 1e-3) / 1e9,
                              "pct_hbm_peak": 100.0 * step_bytes / (ms_f * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                              "attn_tokens_per_s": B / (ms_f * 1e-3),
                              "launches": "per layer pz_decode_attn_append (+ pz_decode_attn_splitk_reduce): 54 per step"}
    if not light:
        graph = capture(torch, model.step)                            # all 90 launches of the step in one HIP graph
        ms_g = time_graphs(torch, [graph], steps, warmup)
        result["hip_graph"] = {"ms_per_step": ms_g, "GBps": step_bytes / (ms_g * 1e-3) / 1e9,
                               "pct_hbm_peak": 100.0 * step_bytes / (ms_g * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                               "attn_tokens_per_s": B / (ms_g * 1e-3)}
        del graph
    if cpu_seqs > 0:
        import oracle
        n_seq = min(cpu_seqs, B)
        tot_t, tot_b, worst, cores = 0.0, 0.0, 0.0, 0
        for w in (128, 8192, 0):
            ls = [l for l in model.layers if l.window == w]
            l0 = next(l for l in ls if l.lay.k_ctx is not None)
            l0.out.fill_(float("nan"))
            l0.step()
            torch.cuda.synchronize()
            got = l0.out[:n_seq].cpu().numpy()
            base, _, want64 = cpu_baseline(pz, wl, oracle, torch, l0, n_seq)
            rms = float(np.sqrt(np.mean(want64.astype(np.float64) ** 2)))
            worst = max(worst, float(np.max(np.abs(got - want64)) / rms))
            tot_t += len(ls) * base["seconds"]
            tot_b += len(ls) * base["value"] * 1e9 * base["seconds"]
            cores = base["cores"]
            l0.lay.k_ctx = l0.lay.v_ctx = None
        result["cpu_baseline"] = {"value": tot_b / tot_t / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
                                  "seconds_scaled_to_36_layers": tot_t, "parity_max_abs_over_rms": worst,
                                  "sample": "first %d of 32 sequences of one layer of each type (window 128, window "
                                            "8192, full), timed once and weighted by the 18/8/10 layer counts" % n_seq}
    else:
        result["cpu_baseline"] = None
    if not args.no_bf16 and not light:
        del model
        torch.cuda.empty_cache()
        mb = Model(pz, wl, torch, pz.KV_BF16, split_tokens=split5)
        ms_b, _ = time_model(torch, mb, steps, warmup, events=False)
        sb = float(sum(l.step_bytes(wl) for l in mb.layers))
        result["bf16_kv"] = {"ms_per_step": ms_b, "GBps": sb / (ms_b * 1e-3) / 1e9,
                             "attn_tokens_per_s": B / (ms_b * 1e-3), "fp8_speedup_tokens_per_s": ms_b / ms_step}
    return result


# ------------------------------------------------------------------ max calibration of the scales

def run_calib(args, pz, wl, torch, light=False):
    """Max calibration of the KV scales: streaming amax over bf16 K and V (1 Mi tokens x 8 heads x 64
    channels each, i.e. one cfg3 layer's worth of new K/V), then the two scales."""
    steps, warmup = (min(args.steps, 30), min(args.warmup, 5)) if light else (args.steps, args.warmup)
    cpu = args.cpu_seqs is None or args.cpu_seqs > 0
    n = 16 * 65536 * 8 * 64
    g = torch.Generator(device="cuda")
    g.manual_seed(11)
    sets = []
    for _ in range(3):
        k = torch.empty(n, dtype=torch.bfloat16, device="cuda")
        v = torch.empty(n, dtype=torch.bfloat16, device="cuda")
        for t0 in range(0, n, 1 << 26):
            m = min(1 << 26, n - t0)
            k[t0:t0 + m] = torch.randn(m, generator=g, device="cuda").to(torch.bfloat16)
            v[t0:t0 + m] = torch.randn(m, generator=g, device="cuda").to(torch.bfloat16)
        sets.append((k, v))
    amax = torch.zeros(2, dtype=torch.float32, device="cuda")
    scales = torch.zeros(2, dtype=torch.float32, device="cuda")

    def step(i, ev=None):
        k, v = sets[i % len(sets)]
        amax.zero_()
        if ev is not None:
            ev[0].record()
        pz.pz_kv_amax_update(k, v, n, amax)
        if ev is not None:
            ev[1].record()
        pz.pz_kv_scales_from_amax(amax, 1, scales)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for i in range(steps):
        step(i, evs[i])
    torch.cuda.synchronize()
    kern = float(np.mean([a.elapsed_time(b) for a, b in evs]))
    nbytes = 2.0 * n * 2
    result = {"metric": "kv-scale max calibration GB/s (bf16 K and V, 2 x 512 Mi elements)", "value": nbytes / (ms * 1e-3) / 1e9,
              "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms,
              "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16 magnitudes as u16",
              "data": "synthetic", "config": {"workload": "calib: amax over 2 GiB of bf16 K/V + scales (pow2 round-up)"},
              "roofline": {"bound": "hbm", "kernel": "kv_amax_kernel", "achieved": nbytes / (kern * 1e-3) / 1e9,
                           "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": nbytes / (kern * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                           "kernel_us_avg": kern * 1e3, "algorithmic_bytes_per_launch": nbytes, "traffic": None}}
    if cpu:
        import oracle
        m = 1 << 24                                               # bounded sample: 16 Mi elements of each tensor
        kb = sets[0][0][:m].view(torch.int16).cpu().numpy().view(np.uint16)
        vb = sets[0][1][:m].view(torch.int16).cpu().numpy().view(np.uint16)
        t0 = time.perf_counter()
        ak, av = oracle.amax_bf16(kb), oracle.amax_bf16(vb)
        dt = time.perf_counter() - t0
        a2 = torch.zeros(2, dtype=torch.float32, device="cuda")
        pz.pz_kv_amax_update(sets[0][0][:m], sets[0][1][:m], m, a2)
        got = a2.cpu().numpy()
        result["cpu_baseline"] = {"value": 2.0 * m * 2 / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                                  "sample": "first 16 Mi elements of K and of V of tensor set 0",
                                  "parity_exact": bool(got[0] == ak and got[1] == av)}
    else:
        result["cpu_baseline"] = None
    return result


# ------------------------------------------------------------------ prefill attention

def run_prefill(args, pz, wl, torch, light=False):
    """Chunked prefill: batch 8, context 32768, the last 2048 positions of every sequence are queries
    (full attention and window 8192).  Matrix-core bound: 4 * d flop per (query, head, attended position)."""
    cpu = args.cpu_seqs is None or args.cpu_seqs > 0
    B, L, n_new = 8, 32768, 2048
    spec = dict(B=B, L=L, window=0, split_tokens=0, outlier_frac=0.0, seed=6)
    layer = Layer(pz, wl, torch, spec, seed=6, kv_dtype=pz.KV_FP8, keep_context=cpu)
    lay = layer.lay
    g = torch.Generator(device="cuda")
    g.manual_seed(66)
    q = torch.randn((B * n_new, lay.Hq, lay.d), generator=g, device="cuda").to(torch.bfloat16)
    q_start = torch.arange(0, (B + 1) * n_new, n_new, dtype=torch.int32, device="cuda")
    out = torch.empty((B * n_new, lay.Hq, lay.d), dtype=torch.float32, device="cuda")
    results = {}
    steps = 5 if light else max(3, args.steps // 20)
    warm = 2 if light else max(1, args.warmup // 4)
    for window in (0, 8192):
        def call():
            pz.pz_prefill_attn(layer.cache, q, q_start, lay.block_table, layer.max_pages, lay.seq_lens_dev, B, lay.Hq,
                               n_new, lay.sinks, lay.sm_scale, layer.k_scale, layer.v_scale, window, out)
        for _ in range(warm):
            call()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for a, b_ in evs:
            a.record(); call(); b_.record()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        kern = float(np.mean([a.elapsed_time(b_) for a, b_ in evs]))
        pos = L - n_new + np.arange(n_new, dtype=np.int64)
        n_att = (np.minimum(pos + 1, window) if window else pos + 1).sum()
        flops = 4.0 * lay.d * lay.Hq * B * float(n_att)
        results[window] = dict(ms=ms, kern_ms=kern, tflops=flops / (kern * 1e-3) / 1e12, flops=flops,
                               tokens_per_s=B * n_new / (ms * 1e-3))
    r0 = results[0]
    result = {"metric": "prefill-attention TFLOP/s + prompt tokens/s, batch 8 x 2048 new tokens at context 32768, FP8 KV",
              "value": r0["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": steps,
              "warmup": warm, "ms_per_step": r0["ms"], "higher_is_better": True, "scaling": "weak",
              "vs_baseline": None, "dtype": DTYPE, "data": "synthetic",
              "config": {"workload": "prefill: batch 8, context 32768, last 2048 positions are queries, 64 q / 8 KV heads, "
                                     "d=64, paged E4M3 KV, causal + sinks (also window 8192)"},
              "prompt_tokens_per_s": r0["tokens_per_s"],
              "roofline": {"bound": "mfma", "kernel": "prefill_attn_kernel<64,1,3>", "achieved": r0["tflops"],
                           "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": r0["tflops"] / MFMA_BF16_PEAK_TFLOPS,
                           "kernel_us_avg": r0["kern_ms"] * 1e3, "algorithmic_flops_per_launch": r0["flops"],
                           "traffic": None},
              "window_8192": {"ms_per_step": results[8192]["ms"], "TFLOPs": results[8192]["tflops"],
                              "prompt_tokens_per_s": results[8192]["tokens_per_s"]}}
    if cpu:
        import oracle
        kc, vc, bt, _, new_k, new_v, new_slots = oracle_sample(oracle, torch, layer, [0])
        oracle.kv_append(kc, vc, new_k, new_v, new_slots, lay.k_scale, lay.v_scale)
        n_s = 32                                                   # bounded sample: the last 32 queries of sequence 0
        qs = q[n_new - n_s:n_new].view(torch.int16).cpu().numpy().view(np.uint16)
        cores = host_cores()
        call_window = 0
        pz.pz_prefill_attn(layer.cache, q, q_start, lay.block_table, layer.max_pages, lay.seq_lens_dev, B, lay.Hq, n_new,
                           lay.sinks, lay.sm_scale, layer.k_scale, layer.v_scale, call_window, out)
        torch.cuda.synchronize()
        got = out[n_new - n_s:n_new].cpu().numpy()
        t0 = time.perf_counter()
        # the sample as a chunk of its own: the n_s newest positions of sequence 0
        want = oracle.prefill_attn(kc, vc, lay.P, qs, np.array([0, n_s]), bt, lay.seq_lens[:1], lay.sinks.cpu().numpy(),
                                   lay.sm_scale, lay.k_scale, lay.v_scale, call_window, nthreads=cores)
        dt = time.perf_counter() - t0
        fl = 4.0 * lay.d * lay.Hq * float((L - n_s + np.arange(n_s) + 1).sum())
        rms = float(np.sqrt(np.mean(want.astype(np.float64) ** 2)))
        result["cpu_baseline"] = {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
                                  "sample": "the last %d query positions of sequence 0 (all 64 heads, full attention)" % n_s,
                                  "parity_max_abs_over_rms": float(np.max(np.abs(got - want)) / rms)}
    else:
        result["cpu_baseline"] = None
    return result


# ------------------------------------------------------------------ bounded window cache through the page pool

def run_pool(args, pz, wl, torch, light=False):
    """A window-8192 layer decoded token by token through the host page pool that recycles the pages
    before each sequence's window: what a sequence holds stays at the window's pages however long it
    grows, which is the memory that lets one GPU hold a larger batch.  Reports the host time of the
    pool per step, the pages held, and the step time; the last step is checked against the oracle on the
    unbounded history of two sequences."""
    B, Hq, Hkv, d, P, W, split = 32, 64, 8, 64, 64, 8192, 1024
    n_steps = 2 * 8192 + 256 if not light else 8192 + 2048
    cpu = args.cpu_seqs is None or args.cpu_seqs > 0
    per_seq = pz.pz_window_pages(W, P)
    max_pages = n_steps // P + 1
    pool = pz.PagePool(B * per_seq, P, B, max_pages, window=W)
    cache = pz.PagedCache.allocate(B * per_seq, P, Hkv, d, pz.KV_FP8, "cuda", fill=0x7F)
    bt_dev = torch.full((B, max_pages), -1, dtype=torch.int32, device="cuda")
    g = torch.Generator(device="cuda")
    g.manual_seed(21)
    k_all = torch.randn((n_steps, B, Hkv, d), generator=g, device="cuda").to(torch.bfloat16)
    v_all = torch.randn((n_steps, B, Hkv, d), generator=g, device="cuda").to(torch.bfloat16)
    q = torch.randn((B, Hq, d), generator=g, device="cuda").to(torch.bfloat16)
    sinks = torch.randn((Hq,), generator=g, device="cuda")
    k_scale = float(np.float32(k_all.abs().max().float().item()) / np.float32(448.0))
    v_scale = float(np.float32(v_all.abs().max().float().item()) / np.float32(448.0))
    S = pz.pz_decode_attn_n_splits(n_steps, W, split)
    wsb = pz.pz_decode_attn_workspace_bytes(B, Hq, d, S)
    ws = torch.empty((wsb // 4,), dtype=torch.float32, device="cuda")
    out = torch.empty((B, Hq, d), dtype=torch.float32, device="cuda")
    lens = torch.zeros((B,), dtype=torch.int32, device="cuda")
    slots_pin = torch.empty((B,), dtype=torch.int64).pin_memory()
    slots_np = slots_pin.numpy()                       # the same memory, written without torch's indexing
    slots_dev = torch.empty((B,), dtype=torch.int64, device="cuda")
    host_s, held_max, n_updates = 0.0, 0, 0
    torch.cuda.synchronize()
    t_all = time.perf_counter()
    for t in range(n_steps):
        t0 = time.perf_counter()
        for b in range(B):
            slots_np[b] = pool.append(b)
        idx, val = pool.drain_updates()
        host_s += time.perf_counter() - t0
        if len(idx):
            n_updates += len(idx)
            bt_dev.view(-1)[torch.from_numpy(idx.astype(np.int64)).to("cuda")] = torch.from_numpy(val).to("cuda")
        slots_dev.copy_(slots_pin)
        torch.cuda.current_stream().synchronize()       # the pinned staging buffer is rewritten next step
        lens.add_(1)
        pz.pz_kv_append_fp8(cache, k_all[t], v_all[t], slots_dev, B, k_scale, v_scale)
        pz.pz_decode_attn(cache, q, bt_dev, max_pages, lens, B, Hq, sinks, 0.125, k_scale, v_scale, W, split, S, ws,
                          wsb, out)
        pz.pz_decode_attn_splitk_reduce(ws, wsb, B, Hq, d, S, lens, W, split, sinks, v_scale, out)
        if t % 512 == 511:
            held_max = max(held_max, int((pool.block_table() >= 0).sum(axis=1).max()))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_all
    held = (pool.block_table() >= 0).sum(axis=1)
    held_max = max(held_max, int(held.max()))
    unbounded = -(-n_steps // P)
    result = {"metric": "bounded window cache: pages held per sequence and host us per step of the page pool (window 8192, B=32)",
              "value": host_s / n_steps * 1e6, "unit": "us of host time per decode step (32 pz_page_pool_append + drain, through ctypes)",
              "n_gpus": 1, "steps": n_steps, "warmup": 0, "ms_per_step": wall / n_steps * 1e3, "higher_is_better": False,
              "scaling": "weak", "vs_baseline": None, "dtype": DTYPE, "data": "synthetic",
              "config": {"workload": "pool: window-8192 layer, batch 32, %d decode steps from an empty cache through "
                                     "pz_page_pool_* (page 64), split-K 1024; block-table updates mirrored to the device" % n_steps},
              "pages_held_per_sequence_max": held_max, "pages_bound_pz_window_pages": per_seq,
              "pages_of_the_unbounded_history": unbounded, "block_table_updates": n_updates,
              "kv_bytes_held_per_sequence": held_max * P * 1024,
              "batch_capacity_factor_at_131072_tokens": (131072 // P) / per_seq,
              "roofline": None}
    pool.close()
    if cpu:
        import oracle
        seqs = [0, B - 1]
        kb = k_all[:, seqs].permute(1, 0, 2, 3).contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        vb = v_all[:, seqs].permute(1, 0, 2, 3).contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        kc, vc = oracle.new_cache(len(seqs) * max_pages * P, Hkv, d)
        obt = (np.arange(len(seqs))[:, None] * max_pages + np.arange(max_pages)[None, :]).astype(np.int32)
        for i in range(len(seqs)):
            oslots = obt[i, np.arange(n_steps) // P].astype(np.int64) * P + np.arange(n_steps) % P
            oracle.kv_append(kc, vc, kb[i], vb[i], oslots, k_scale, v_scale)
        qs = q[seqs].view(torch.int16).cpu().numpy().view(np.uint16)
        want = oracle.decode_attn(kc, vc, P, qs, obt, np.full(len(seqs), n_steps, dtype=np.int32), sinks.cpu().numpy(),
                                  0.125, k_scale, v_scale, W, accum="f64", nthreads=host_cores())
        got = out[seqs].cpu().numpy()
        rms = float(np.sqrt(np.mean(want.astype(np.float64) ** 2)))
        result["cpu_baseline"] = {"value": None, "unit": "", "cores": host_cores(), "kind": "oracle",
                                  "sample": "the last step's rows of sequences 0 and 31 against the oracle on their whole, "
                                            "unbounded history", "parity_max_abs_over_rms": float(np.max(np.abs(got - want)) / rms)}
    else:
        result["cpu_baseline"] = None
    return result


# ------------------------------------------------------------------ fused rotary + append

def run_rope(args, pz, wl, torch, light=False):
    """pz_rope_kv_append_fp8 (rotary embedding of q and k, quantise, append: one launch) against
    pz_kv_append_fp8 alone at decode sizes: what the rotation costs when it rides in the append launch."""
    cpu = args.cpu_seqs is None or args.cpu_seqs > 0
    Hq, Hkv, d, P = 64, 8, 64, 64
    n_pos = 131072
    cos, sin = pz.pz_rope_yarn_table(pz.YarnParams(), d, n_pos)
    cd, sd = torch.from_numpy(cos).to("cuda"), torch.from_numpy(sin).to("cuda")
    g = torch.Generator(device="cuda")
    g.manual_seed(31)
    reps = 200 if light else 1000
    rows = {}
    first = None
    for B in (16, 32, 64, 128, 256):
        num_pages = B + 4
        cache = pz.PagedCache.allocate(num_pages, P, Hkv, d, pz.KV_FP8, "cuda", fill=0)
        q = torch.randn((B, Hq, d), generator=g, device="cuda").to(torch.bfloat16)
        k = torch.randn((B, Hkv, d), generator=g, device="cuda").to(torch.bfloat16)
        v = torch.randn((B, Hkv, d), generator=g, device="cuda").to(torch.bfloat16)
        q_out = torch.empty_like(q)
        rng = np.random.default_rng(B)
        pos_h = rng.integers(0, n_pos, B).astype(np.int32)
        slots_h = (np.arange(B, dtype=np.int64) * P + pos_h % P)
        pos, slots = torch.from_numpy(pos_h).to("cuda"), torch.from_numpy(slots_h).to("cuda")
        ks, vs = 6.0 / 448, 5.0 / 448

        def timed(fn):
            """us per call on the GPU: 50 calls recorded into a HIP graph, replays timed (calls issued one by one
            from Python are bound by the interpreter, about 7 us each)."""
            def fifty():
                for _ in range(50):
                    fn()
            graph = capture(torch, fifty)
            for _ in range(3):
                graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(max(1, reps // 50)):
                graph.replay()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / (max(1, reps // 50) * 50) * 1e6

        us_rope = timed(lambda: pz.pz_rope_kv_append_fp8(cache, q, q_out, k, v, pos, cd, sd, slots, B, Hq, ks, vs))
        us_plain = timed(lambda: pz.pz_kv_append_fp8(cache, k, v, slots, B, ks, vs))
        rows["B=%d" % B] = {"rope_kv_append_us": us_rope, "kv_append_us": us_plain}
        if first is None:
            first = (cache, q, k, v, q_out, pos_h, slots_h, ks, vs, B)
    result = {"metric": "fused rotary (YaRN factor 56) + quantise-and-append, us per call at decode sizes",
              "value": rows["B=16"]["rope_kv_append_us"], "unit": "us per call (B=16)", "n_gpus": 1, "steps": reps,
              "warmup": 20, "ms_per_step": rows["B=16"]["rope_kv_append_us"] * 1e-3, "higher_is_better": False,
              "scaling": "weak", "vs_baseline": None, "dtype": "fp32 rotation, bf16 q, e4m3 K/V", "data": "synthetic",
              "config": {"workload": "rope: pz_rope_kv_append_fp8 (64 q + 8 KV heads per token, d=64) against "
                                     "pz_kv_append_fp8 alone, 1 token per sequence, back-to-back launches replayed from a HIP graph"},
              "by_batch": rows, "roofline": None}
    if cpu:
        import oracle
        cache, q, k, v, q_out, pos_h, slots_h, ks, vs, B = first
        pz.pz_rope_kv_append_fp8(cache, q, q_out, k, v, torch.from_numpy(pos_h).to("cuda"), cd, sd,
                                 torch.from_numpy(slots_h).to("cuda"), B, Hq, ks, vs)
        torch.cuda.synchronize()
        ocos, osin = oracle.yarn_table(d, n_pos)
        bits = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
        okc, ovc = oracle.new_cache(cache.num_pages * P, Hkv, d)
        oq = oracle.rope_kv_append(okc, ovc, bits(q), bits(k), bits(v), pos_h, ocos, osin, slots_h, ks, vs)
        gk = cache.k.permute(0, 2, 1, 3).reshape(-1, Hkv, d).cpu().numpy()
        same_rows = np.all(ocos[pos_h] == cos[pos_h], axis=1) & np.all(osin[pos_h] == sin[pos_h], axis=1)
        result["cpu_baseline"] = {"value": None, "unit": "", "cores": 1, "kind": "oracle",
                                  "sample": "the B=16 call: q bits and K cache bytes of the tokens whose table rows agree "
                                            "bit for bit between the library's and the oracle's table (%d of %d)"
                                            % (int(same_rows.sum()), B),
                                  "parity_exact": bool(np.array_equal(bits(q_out)[same_rows], oq[same_rows]) and
                                                       np.array_equal(gk[slots_h[same_rows]], okc[slots_h[same_rows]]))}
    else:
        result["cpu_baseline"] = None
    return result


# ------------------------------------------------------------------ driver

def run_workload(args, pz, wl, torch, name, light=False):
    if name in WORKLOADS:
        return run_layer_workload(args, pz, wl, torch, name, light)
    return {"cfg5": run_cfg5, "calib": run_calib, "prefill": run_prefill, "pool": run_pool, "rope": run_rope}[name](
        args, pz, wl, torch, light)


def condensed(r):
    """What `all_configs` keeps of a workload's result."""
    keep = {"metric": r["metric"], "value": r["value"], "unit": r["unit"], "ms_per_step": r["ms_per_step"],
            "steps": r["steps"], "workload": r["config"]["workload"]}
    for key in ("attn_tokens_per_s", "pct_hbm_peak", "prompt_tokens_per_s", "by_batch", "pages_held_per_sequence_max",
                "pages_bound_pz_window_pages", "pages_of_the_unbounded_history", "batch_capacity_factor_at_131072_tokens"):
        if key in r:
            keep[key] = r[key]
    if r.get("roofline"):
        rf = r["roofline"]
        keep["roofline"] = {k: rf[k] for k in ("bound", "kernel", "achieved", "peak", "unit", "frac", "kernel_us_avg",
                                               "algorithmic_bytes_per_launch", "algorithmic_flops_per_launch") if k in rf}
    if r.get("fused_append"):
        keep["fused_append_ms_per_step"] = r["fused_append"]["ms_per_step"]
    if r.get("cpu_baseline"):
        cb = r["cpu_baseline"]
        keep["oracle"] = {k: cb[k] for k in ("parity_max_abs_over_rms", "parity_exact", "sample", "cores", "value", "unit")
                          if k in cb}
    return keep


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default=None, choices=sorted(WORKLOADS) + OTHER_WORKLOADS,
                    help="one workload in full; without it: cfg3 in full plus `all_configs`")
    ap.add_argument("--no-all-configs", action="store_true", help="default run without the `all_configs` part")
    ap.add_argument("--cpu-seqs", type=int, default=None,
                    help="sequences in the oracle's sample (0 = skip; default: the whole batch on cfg3 / cfg2, a few otherwise)")
    ap.add_argument("--no-bf16", action="store_true", help="skip the BF16-KV comparison run")
    ap.add_argument("--split-tokens", type=int, default=None, help="override the workload's split-K chunk length")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 768 MiB device-to-device copy (reference for HBM traffic counters)")
    ap.add_argument("--source-hash", action="store_true", help="print the hash of the decode-attention kernel sources and exit")
    args = ap.parse_args()
    if args.source_hash:
        print(kernel_source_hash())
        return
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU (the decode-attention path needs no collective: it shards over KV heads or sequences): "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2602_11937_amd as pz
    import workloads as wl
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    pz.lib()                                                      # fails loudly if libpz.so is not built
    torch.cuda.set_device(0)
    if args.workload is not None:
        print(json.dumps(run_workload(args, pz, wl, torch, args.workload)), flush=True)
        return
    t0 = time.perf_counter()
    result = run_workload(args, pz, wl, torch, "cfg3")
    log("cfg3 done after %.0f s" % (time.perf_counter() - t0))
    if not args.no_all_configs:
        result["all_configs"] = {}
        for name in ALL_CONFIGS:
            torch.cuda.empty_cache()
            result["all_configs"][name] = condensed(run_workload(args, pz, wl, torch, name, light=True))
            log("%s done after %.0f s" % (name, time.perf_counter() - t0))
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
