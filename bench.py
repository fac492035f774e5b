#!/usr/bin/env python3
"""Benchmark of the decode-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3|cfg2|cfg4_w128|cfg4_w8192|cfg5]

A step is one pass of the whole path over one batch: quantise-and-append of one new token per
sequence, decode attention (split-K partials + log-sum-exp merge, or single pass for short
windows), all through the C ABI.  Inputs are seeded synthetic gpt-oss-shaped tensors, resident
in HBM before the timed region.  Consecutive steps walk over several independent cache
instances so that no step re-reads data the 256 MB Infinity Cache may still hold.

Prints ONE JSON line: metric / value (algorithmic GB/s of the whole step) / ms_per_step, `roofline`
(the dominant kernel: algorithmic bytes per launch over its event-timed duration, against the 8 TB/s
HBM peak, plus the HBM traffic measured with hardware counters), `cpu_baseline` (the CPU oracle timed
on a bounded sample of the same workload, with a parity figure), `bf16_kv` (the same step on a BF16
cache), `repetitions` (spread of the step time over four timed regions), `fused_append` (the step with
the append fused into the attention launch), `stream_read` (the box's plain streaming-read rate over
the same cache bytes, measured in the same run), `hip_graph` (the step replayed from a HIP graph) and
`tuned_split` (the same step with longer split-K chunks).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

# HBM bytes per decode_attn launch from rocprofv3 FETCH_SIZE + WRITE_SIZE (profiles/decode_step_cfg3_fp8_hbm_traffic.txt:
# counters scaled by what they read for a plain 768 MiB copy); only measured for the default cfg3 launch.
MEASURED_TRAFFIC_BYTES = {"cfg3": 1078362834}

METRIC = "decode-attention GB/s (% of HBM peak) + attn tokens/s, B=16 ctx=64K FP8 KV"
HBM_PEAK_GBPS = 8000.0
CFG5_SPLIT = 8192      # split-K chunk length of cfg5's full and window-8192 layers (the configuration names none;
                       # 8192 measured best: 1024 4.17 ms, 2048 4.03, 4096 3.81, 8192 3.77, 16384 4.11)

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
    # single layers of the heterogeneous step (cfg5), for tests and tuning
    "cfg5_full": dict(B=32, L=(1024, 131072), window=0, split_tokens=CFG5_SPLIT, outlier_frac=0.0, seed=5, instances=3,
                      bounded=True, text="cfg5 full-attention layer: batch 32, ragged contexts U[1024,131072], split-K %d" % CFG5_SPLIT),
    "cfg5_w8192": dict(B=32, L=(1024, 131072), window=8192, split_tokens=CFG5_SPLIT, outlier_frac=0.0, seed=5, instances=3,
                       bounded=True, text="cfg5 window-8192 layer: batch 32, ragged contexts U[1024,131072], split-K %d" % CFG5_SPLIT),
    "cfg5_w128": dict(B=32, L=(1024, 131072), window=128, split_tokens=0, outlier_frac=0.0, seed=5, instances=3,
                      bounded=True, text="cfg5 window-128 layer: batch 32, ragged contexts U[1024,131072], single pass"),
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Layer:
    """One cache instance + everything a step on it needs, with the C-ABI arguments prepared."""

    def __init__(self, pz, wl, torch, spec, seed, kv_dtype, keep_context=False):
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
        lay = wl.device_layer(B=B, seq_lens=seq_lens, window=self.window, seed=seed,
                              outlier_frac=spec["outlier_frac"], resident=resident)
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
        self.set_split(self.split)

    def set_split(self, split_tokens):
        """(Re)size the split-K workspace for a chunk length (0 = single pass)."""
        pz, lay = self.pz, self.lay
        self.split = split_tokens
        self.S = pz.pz_decode_attn_n_splits(int(lay.seq_lens.max()), self.window, self.split) if self.split else 0
        self.ws_bytes = pz.pz_decode_attn_workspace_bytes(lay.B, lay.Hq, lay.d, self.S) if self.split else 0
        self.ws = self.torch.empty((max(self.ws_bytes, 4) // 4,), dtype=self.torch.float32, device="cuda")

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
        self.pz.pz_kv_append_fp8(self.cache, lay.k_new, lay.v_new, lay.new_slots, lay.B, self.k_scale, self.v_scale)

    def attn(self):
        lay, pz = self.lay, self.pz
        pz.pz_decode_attn(self.cache, lay.q, lay.block_table, self.max_pages, lay.seq_lens_dev, lay.B, lay.Hq,
                          lay.sinks, lay.sm_scale, self.k_scale, self.v_scale, self.window, self.split, self.S,
                          self.ws if self.split else None, self.ws_bytes, self.out)

    def attn_append(self):
        """The append of the step's new token fused into the attention launch."""
        lay, pz = self.lay, self.pz
        pz.pz_decode_attn_append(self.cache, lay.k_new, lay.v_new, lay.q, lay.block_table, self.max_pages,
                                 lay.seq_lens_dev, lay.B, lay.Hq, lay.sinks, lay.sm_scale, self.k_scale, self.v_scale,
                                 self.window, self.split, self.S, self.ws if self.split else None, self.ws_bytes,
                                 self.out)

    def step_fused(self):
        self.attn_append()
        self.reduce()

    def reduce(self):
        if not self.split:
            return
        lay, pz = self.lay, self.pz
        pz.pz_decode_attn_splitk_reduce(self.ws, self.ws_bytes, lay.B, lay.Hq, lay.d, self.S, lay.seq_lens_dev,
                                        self.window, self.split, lay.sinks, self.v_scale, self.out)

    def step(self, ev=None):
        self.append()
        if ev is not None:
            ev[0].record()
        self.attn()
        if ev is not None:
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
    off, fp = lay.ctx_offsets, lay.first_pos
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
        kb = lay.k_ctx[off[b]:off[b + 1]].view(torch.int16).cpu().numpy().view(np.uint16)
        vb = lay.v_ctx[off[b]:off[b + 1]].view(torch.int16).cpu().numpy().view(np.uint16)
        j = np.arange(int(fp[b]), int(lay.seq_lens[b]), dtype=np.int64)
        slots = bt[i, j // P].astype(np.int64) * P + j % P
        oracle.kv_append(kc, vc, kb[:-1], vb[:-1], slots[:-1], lay.k_scale, lay.v_scale)
        new_k.append(kb[-1:]); new_v.append(vb[-1:]); new_slots.append(slots[-1:])
    q = lay.q[torch.as_tensor(list(seqs), device=lay.q.device)].view(torch.int16).cpu().numpy().view(np.uint16)
    return kc, vc, bt, q, np.concatenate(new_k), np.concatenate(new_v), np.concatenate(new_slots)


def cpu_baseline(pz, wl, oracle, torch, layer, n_seq):
    """The oracle, as it stands, on the first n_seq sequences of a Layer (all query heads): its
    own quantise-and-append of their context (set-up, untimed), then timed: append of the new
    tokens + unsplit attention.  Returns the baseline dict and the oracle rows."""
    lay = layer.lay
    cores = min(len(os.sched_getaffinity(0)), 16)
    seqs = list(range(n_seq))
    kc, vc, bt, q, new_k, new_v, new_slots = oracle_sample(oracle, torch, layer, seqs)
    sinks = lay.sinks.cpu().numpy()
    t0 = time.perf_counter()
    oracle.kv_append(kc, vc, new_k, new_v, new_slots, lay.k_scale, lay.v_scale)
    want = oracle.decode_attn(kc, vc, lay.P, q, bt, lay.seq_lens[:n_seq], sinks, lay.sm_scale, lay.k_scale,
                              lay.v_scale, layer.window, nthreads=cores)
    dt = time.perf_counter() - t0
    toks = wl.kv_tokens_read(lay.seq_lens[:n_seq], layer.window)
    nbytes = toks * wl.kv_bytes_per_token(lay.Hkv, lay.d, 1)
    base = {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
            "seconds": dt, "attn_tokens_per_s": n_seq / dt,
            "sample": "first %d of %d sequences of cache instance 0, all %d query heads: oracle kv_append of "
                      "their new tokens + unsplit fp32 decode attention (%d cached tokens)"
                      % (n_seq, lay.B, lay.Hq, toks)}
    return base, want


class Model:
    """The heterogeneous 36-layer decode step: every layer appends one token per sequence and runs
    its attention (window 128: single pass; window 8192 and full: split-K with `split_tokens`-long chunks + merge)."""

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


def run_cfg5(args, pz, wl, torch):
    """36 layers: 18 x window 128, 8 x window 8192, 10 x full; batch 32, contexts U[1024,131072]."""
    text = ("cfg5: 36-layer decode step (18 x window-128, 8 x window-8192, 10 x full attention), batch 32, ragged "
            "contexts U[1024,131072], 64 q / 8 KV heads, d=64, paged E4M3 KV with per-layer K/V scales; every layer "
            "= kv_append of 1 token/seq + decode attention (+ LSE merge; split-K chunks of %d tokens)" % (
                args.split_tokens if args.split_tokens is not None else CFG5_SPLIT))
    t0 = time.perf_counter()
    split5 = args.split_tokens if args.split_tokens is not None else CFG5_SPLIT
    model = Model(pz, wl, torch, pz.KV_FP8, keep_context_types=(128, 8192, 0) if args.cpu_seqs > 0 else (),
                  split_tokens=split5)
    log("built the 36 FP8 layer caches in %.1f s" % (time.perf_counter() - t0))
    ms_step, _ = time_model(torch, model, args.steps, args.warmup, events=False)
    reps = [ms_step] + [time_model(torch, model, args.steps, 1, events=False)[0] for _ in range(3)]
    ms_ev, kern = time_model(torch, model, args.steps, args.warmup, events=True)
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
        "value": step_bytes / (ms_step * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "e4m3 KV -> bf16 MFMA operands, f32 accumulate", "data": "synthetic",
        "config": {"workload": text, "batch": B, "layers": by_type},
        "attn_tokens_per_s": B / (ms_step * 1e-3),
        "pct_hbm_peak": 100.0 * step_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "repetitions": {"n": len(reps), "ms_per_step_mean": float(np.mean(reps)), "ms_per_step_std": float(np.std(reps))},
        "roofline": {"bound": "hbm", "kernel": "decode_attn_balanced_kernel<64,1> (the 10 full-attention layers)",
                     "achieved": full_bytes / (kern_avg * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": full_bytes / (kern_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS, "kernel_us_avg": kern_avg * 1e3,
                     "ms_per_step_with_events": ms_ev, "algorithmic_bytes_per_launch": full_bytes, "traffic": None},
    }
    ms_f = time_model_fused(torch, model, args.steps, args.warmup)
    result["fused_append"] = {"ms_per_step": ms_f, "GBps": step_bytes / (ms_f * 1e-3) / 1e9,
                              "pct_hbm_peak": 100.0 * step_bytes / (ms_f * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                              "attn_tokens_per_s": B / (ms_f * 1e-3),
                              "launches": "per layer pz_decode_attn_append (+ pz_decode_attn_splitk_reduce): 54 per step"}
    graph = capture(torch, model.step)                            # all 90 launches of the step in one HIP graph
    ms_g = time_graphs(torch, [graph], args.steps, args.warmup)
    result["hip_graph"] = {"ms_per_step": ms_g, "GBps": step_bytes / (ms_g * 1e-3) / 1e9,
                           "pct_hbm_peak": 100.0 * step_bytes / (ms_g * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                           "attn_tokens_per_s": B / (ms_g * 1e-3)}
    del graph
    if args.cpu_seqs > 0:
        import oracle
        n_seq = min(args.cpu_seqs, B)
        tot_t, tot_b, worst, cores = 0.0, 0.0, 0.0, 0
        for w in (128, 8192, 0):
            ls = [l for l in model.layers if l.window == w]
            l0 = next(l for l in ls if l.lay.k_ctx is not None)
            l0.step()
            torch.cuda.synchronize()
            got = l0.out[:n_seq].cpu().numpy()
            base, want = cpu_baseline(pz, wl, oracle, torch, l0, n_seq)
            rms = float(np.sqrt(np.mean(want.astype(np.float64) ** 2)))
            worst = max(worst, float(np.max(np.abs(got - want)) / rms))
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
    if not args.no_bf16:
        del model
        torch.cuda.empty_cache()
        mb = Model(pz, wl, torch, pz.KV_BF16, split_tokens=split5)
        ms_b, _ = time_model(torch, mb, args.steps, args.warmup, events=False)
        sb = float(sum(l.step_bytes(wl) for l in mb.layers))
        result["bf16_kv"] = {"ms_per_step": ms_b, "GBps": sb / (ms_b * 1e-3) / 1e9,
                             "attn_tokens_per_s": B / (ms_b * 1e-3), "fp8_speedup_tokens_per_s": ms_b / ms_step}
    print(json.dumps(result), flush=True)


def run_calib(args, pz, wl, torch):
    """Max calibration of the KV scales: streaming amax over bf16 K and V (1 Mi tokens x 8 heads x 64
    channels each, i.e. one cfg3 layer's worth of new K/V), then the two scales."""
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

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for i in range(args.steps):
        step(i, evs[i])
    torch.cuda.synchronize()
    kern = float(np.mean([a.elapsed_time(b) for a, b in evs]))
    nbytes = 2.0 * n * 2
    result = {"metric": "kv-scale max calibration GB/s (bf16 K and V, 2 x 512 Mi elements)", "value": nbytes / (ms * 1e-3) / 1e9,
              "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
              "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16 magnitudes as u16",
              "data": "synthetic", "config": {"workload": "calib: amax over 2 GiB of bf16 K/V + scales (pow2 round-up)"},
              "roofline": {"bound": "hbm", "kernel": "kv_amax_kernel", "achieved": nbytes / (kern * 1e-3) / 1e9,
                           "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": nbytes / (kern * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                           "kernel_us_avg": kern * 1e3, "algorithmic_bytes_per_launch": nbytes, "traffic": None}}
    if args.cpu_seqs > 0:
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
    print(json.dumps(result), flush=True)


def run_prefill(args, pz, wl, torch):
    """Chunked prefill: batch 8, context 32768, the last 2048 positions of every sequence are queries
    (full attention and window 8192).  Matrix-core bound: 4 * d flop per (query, head, attended position)."""
    B, L, n_new = 8, 32768, 2048
    spec = dict(B=B, L=L, window=0, split_tokens=0, outlier_frac=0.0, seed=6)
    layer = Layer(pz, wl, torch, spec, seed=6, kv_dtype=pz.KV_FP8, keep_context=args.cpu_seqs > 0)
    lay = layer.lay
    g = torch.Generator(device="cuda")
    g.manual_seed(66)
    q = torch.randn((B * n_new, lay.Hq, lay.d), generator=g, device="cuda").to(torch.bfloat16)
    q_start = torch.arange(0, (B + 1) * n_new, n_new, dtype=torch.int32, device="cuda")
    out = torch.empty((B * n_new, lay.Hq, lay.d), dtype=torch.float32, device="cuda")
    results = {}
    for window in (0, 8192):
        def call():
            pz.pz_prefill_attn(layer.cache, q, q_start, lay.block_table, layer.max_pages, lay.seq_lens_dev, B, lay.Hq,
                               n_new, lay.sinks, lay.sm_scale, layer.k_scale, layer.v_scale, window, out)
        for _ in range(max(1, args.warmup // 4)):
            call()
        steps = max(3, args.steps // 20)
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
              "value": r0["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": max(3, args.steps // 20),
              "warmup": max(1, args.warmup // 4), "ms_per_step": r0["ms"], "higher_is_better": True, "scaling": "weak",
              "vs_baseline": None, "dtype": "e4m3 KV -> bf16 MFMA operands, f32 accumulate", "data": "synthetic",
              "config": {"workload": "prefill: batch 8, context 32768, last 2048 positions are queries, 64 q / 8 KV heads, "
                                     "d=64, paged E4M3 KV, causal + sinks (also window 8192)"},
              "prompt_tokens_per_s": r0["tokens_per_s"],
              "roofline": {"bound": "mfma", "kernel": "prefill_attn_kernel<64,1,3>", "achieved": r0["tflops"],
                           "peak": 2500.0, "unit": "TFLOP/s", "frac": r0["tflops"] / 2500.0,
                           "kernel_us_avg": r0["kern_ms"] * 1e3, "algorithmic_flops_per_launch": r0["flops"],
                           "traffic": None},
              "window_8192": {"ms_per_step": results[8192]["ms"], "TFLOPs": results[8192]["tflops"],
                              "prompt_tokens_per_s": results[8192]["tokens_per_s"]}}
    if args.cpu_seqs > 0:
        import oracle
        kc, vc, bt, _, new_k, new_v, new_slots = oracle_sample(oracle, torch, layer, [0])
        oracle.kv_append(kc, vc, new_k, new_v, new_slots, lay.k_scale, lay.v_scale)
        n_s = 32                                                   # bounded sample: the last 32 queries of sequence 0
        qs = q[n_new - n_s:n_new].view(torch.int16).cpu().numpy().view(np.uint16)
        cores = min(len(os.sched_getaffinity(0)), 16)
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
    print(json.dumps(result), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="cfg3", choices=sorted(WORKLOADS) + ["cfg5", "calib", "prefill"])
    ap.add_argument("--cpu-seqs", type=int, default=4, help="sequences in the oracle's bounded sample (0 = skip)")
    ap.add_argument("--no-bf16", action="store_true", help="skip the BF16-KV comparison run")
    ap.add_argument("--split-tokens", type=int, default=None, help="override the workload's split-K chunk length")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 768 MiB device-to-device copy (reference for HBM traffic counters)")
    args = ap.parse_args()
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
    if args.workload == "cfg5":
        return run_cfg5(args, pz, wl, torch)
    if args.workload == "calib":
        return run_calib(args, pz, wl, torch)
    if args.workload == "prefill":
        return run_prefill(args, pz, wl, torch)
    spec = dict(WORKLOADS[args.workload])
    if args.split_tokens is not None:
        spec["split_tokens"] = args.split_tokens
        spec["text"] += " [split_tokens overridden to %d]" % args.split_tokens
    torch.cuda.set_device(0)

    if args.calib_copy:
        src = torch.ones((768 << 20) // 4, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    t_setup = time.perf_counter()
    layers = [Layer(pz, wl, torch, spec, seed=spec["seed"] + 1000 * r, kv_dtype=pz.KV_FP8,
                    keep_context=(r == 0 and args.cpu_seqs > 0)) for r in range(spec["instances"])]
    log("built %d FP8 cache instances in %.1f s" % (len(layers), time.perf_counter() - t_setup))
    ms_step, _ = time_steps(torch, layers, args.steps, args.warmup, events=False)
    # three more timed regions of the same K steps: spread of the step time between repetitions
    reps = [ms_step] + [time_steps(torch, layers, args.steps, 2, events=False)[0] for _ in range(3)]
    ms_step_ev, kern_ms = time_steps(torch, layers, args.steps, args.warmup, events=True)
    attn_bytes = float(np.mean([l.attn_bytes(wl) for l in layers]))
    step_bytes = float(np.mean([l.step_bytes(wl) for l in layers]))
    B = spec["B"]
    kern_avg_ms = float(kern_ms.mean())
    result = {
        "metric": METRIC if args.workload == "cfg3" else METRIC.split(", B=16")[0] + ", " + args.workload + " FP8 KV",
        "value": step_bytes / (ms_step * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "e4m3 KV -> bf16 MFMA operands, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": spec["text"], "batch": B, "n_q_heads": 64, "n_kv_heads": 8, "head_dim": 64,
                   "page_size": 64, "window": spec["window"], "split_tokens": spec["split_tokens"],
                   "cache_instances_rotated": len(layers)},
        "attn_tokens_per_s": B / (ms_step * 1e-3),
        "pct_hbm_peak": 100.0 * step_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "repetitions": {"n": len(reps), "ms_per_step_mean": float(np.mean(reps)), "ms_per_step_std": float(np.std(reps))},
        "roofline": {"bound": "hbm", "kernel": ("decode_attn_balanced_kernel<64,1>" if spec["window"] == 0 and
                                                spec["split_tokens"] > 0 else "decode_attn_kernel<64,1>"),
                     "achieved": attn_bytes / (kern_avg_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": attn_bytes / (kern_avg_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "kernel_us_avg": kern_avg_ms * 1e3, "kernel_us_std": float(kern_ms.std() * 1e3),
                     "ms_per_step_with_events": ms_step_ev,
                     "algorithmic_bytes_per_launch": attn_bytes,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(args.workload) if args.split_tokens is None else None},
    }
    ms_f = time_fused(torch, layers, args.steps, args.warmup)
    result["fused_append"] = {"ms_per_step": ms_f, "GBps": step_bytes / (ms_f * 1e-3) / 1e9,
                              "pct_hbm_peak": 100.0 * step_bytes / (ms_f * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                              "attn_tokens_per_s": B / (ms_f * 1e-3),
                              "launches": "pz_decode_attn_append + pz_decode_attn_splitk_reduce"
                              if spec["split_tokens"] else "pz_decode_attn_append"}
    # the box's plain streaming-read rate over the very same cache bytes: the library's amax kernel
    # (16-byte loads, a max per element, nothing written) run over the K and V arrays of each instance
    if args.workload in ("cfg3", "cfg2"):
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
    # the same step launched as one replay of a recorded HIP graph (one graph per cache instance)
    graphs = [capture(torch, l.step) for l in layers]
    ms_g = time_graphs(torch, graphs, args.steps, args.warmup)
    result["hip_graph"] = {"ms_per_step": ms_g, "GBps": step_bytes / (ms_g * 1e-3) / 1e9,
                           "pct_hbm_peak": 100.0 * step_bytes / (ms_g * 1e-3) / 1e9 / HBM_PEAK_GBPS}
    del graphs
    if args.workload == "cfg3" and args.split_tokens is None:
        # the same step with the chunk length a caller free to choose would use (fewer, longer partials)
        for l in layers:
            l.set_split(8192)
        ms_t, _ = time_steps(torch, layers, args.steps, args.warmup, events=False)
        result["tuned_split"] = {"split_tokens": 8192, "ms_per_step": ms_t, "GBps": step_bytes / (ms_t * 1e-3) / 1e9,
                                 "pct_hbm_peak": 100.0 * step_bytes / (ms_t * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                                 "attn_tokens_per_s": B / (ms_t * 1e-3)}
        for l in layers:
            l.set_split(spec["split_tokens"])

    if args.cpu_seqs > 0:
        import oracle
        n_seq = min(args.cpu_seqs, B)
        layers[0].step()
        torch.cuda.synchronize()
        got = layers[0].out[:n_seq].cpu().numpy()
        base, want = cpu_baseline(pz, wl, oracle, torch, layers[0], n_seq)
        rms = float(np.sqrt(np.mean(want.astype(np.float64) ** 2)))
        base["parity_max_abs_over_rms"] = float(np.max(np.abs(got - want)) / rms)
        result["cpu_baseline"] = base
        layers[0].lay.k_ctx = layers[0].lay.v_ctx = None
    else:
        result["cpu_baseline"] = None

    if not args.no_bf16:
        del layers
        torch.cuda.empty_cache()
        n_inst = max(2, spec["instances"] - 1)
        bl = [Layer(pz, wl, torch, spec, seed=spec["seed"] + 1000 * r, kv_dtype=pz.KV_BF16) for r in range(n_inst)]
        ms_b, _ = time_steps(torch, bl, args.steps, args.warmup, events=False)
        _, kern_b = time_steps(torch, bl, args.steps, args.warmup, events=True)
        sb = float(np.mean([l.step_bytes(wl) for l in bl]))
        ab = float(np.mean([l.attn_bytes(wl) for l in bl]))
        result["bf16_kv"] = {"ms_per_step": ms_b, "GBps": sb / (ms_b * 1e-3) / 1e9,
                             "attn_tokens_per_s": B / (ms_b * 1e-3), "kernel_us_avg": float(kern_b.mean() * 1e3),
                             "kernel_GBps": ab / (float(kern_b.mean()) * 1e-3) / 1e9,
                             "fp8_speedup_tokens_per_s": ms_b / ms_step}
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
