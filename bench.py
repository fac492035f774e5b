#!/usr/bin/env python3
"""Benchmark of the decode-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3|cfg2|cfg4_w128|cfg4_w8192]

A step is one pass of the whole path over one batch: quantise-and-append of one new token per
sequence, decode attention (split-K partials + log-sum-exp merge, or single pass for short
windows), all through the C ABI.  Inputs are seeded synthetic gpt-oss-shaped tensors, resident
in HBM before the timed region.  Consecutive steps walk over several independent cache
instances so that no step re-reads data the 256 MB Infinity Cache may still hold.

Prints ONE JSON line (see the design doc for the field definitions).
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
MEASURED_TRAFFIC_BYTES = {"cfg3": 1091883524}

METRIC = "decode-attention GB/s (% of HBM peak) + attn tokens/s, B=16 ctx=64K FP8 KV"
HBM_PEAK_GBPS = 8000.0

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
        lay = wl.device_layer(B=B, seq_lens=seq_lens, window=self.window, seed=seed,
                              outlier_frac=spec["outlier_frac"])
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


def cpu_baseline(pz, wl, oracle, torch, layer, n_seq):
    """The oracle, as it stands, on the first n_seq sequences of instance 0 (all query heads):
    its own quantise-and-append of their whole context (set-up, untimed), then timed: append of
    the new tokens + unsplit attention.  Returns the baseline dict and the oracle rows."""
    lay = layer.lay
    cores = min(len(os.sched_getaffinity(0)), 16)
    off = np.concatenate([[0], np.cumsum(lay.seq_lens.astype(np.int64))])
    P = lay.P
    n_pages = [-(-int(lay.seq_lens[b]) // P) for b in range(n_seq)]
    bt = np.full((n_seq, max(n_pages)), -1, dtype=np.int32)
    at = 0
    for b in range(n_seq):                                        # compact page numbering for the sample
        bt[b, :n_pages[b]] = np.arange(at, at + n_pages[b])
        at += n_pages[b]
    kc, vc = oracle.new_cache(at * P, lay.Hkv, lay.d, oracle.KV_FP8)
    new_k, new_v, new_slots = [], [], []
    for b in range(n_seq):
        L = int(lay.seq_lens[b])
        kb = lay.k_ctx[off[b]:off[b + 1]].view(torch.int16).cpu().numpy().view(np.uint16)
        vb = lay.v_ctx[off[b]:off[b + 1]].view(torch.int16).cpu().numpy().view(np.uint16)
        j = np.arange(L, dtype=np.int64)
        slots = bt[b, j // P].astype(np.int64) * P + j % P
        oracle.kv_append(kc, vc, kb[:-1], vb[:-1], slots[:-1], lay.k_scale, lay.v_scale)
        new_k.append(kb[-1:]); new_v.append(vb[-1:]); new_slots.append(slots[-1:])
    q = lay.q[:n_seq].view(torch.int16).cpu().numpy().view(np.uint16)
    sinks = lay.sinks.cpu().numpy()
    t0 = time.perf_counter()
    oracle.kv_append(kc, vc, np.concatenate(new_k), np.concatenate(new_v), np.concatenate(new_slots),
                     lay.k_scale, lay.v_scale)
    want = oracle.decode_attn(kc, vc, P, q, bt, lay.seq_lens[:n_seq], sinks, lay.sm_scale, lay.k_scale,
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg3", choices=sorted(WORKLOADS))
    ap.add_argument("--cpu-seqs", type=int, default=4, help="sequences in the oracle's bounded sample (0 = skip)")
    ap.add_argument("--no-bf16", action="store_true", help="skip the BF16-KV comparison run")
    ap.add_argument("--split-tokens", type=int, default=None, help="override the workload's split-K chunk length")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 768 MiB device-to-device copy (reference for HBM traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU (the path needs no collective; see DESIGN.md on sharding): "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2602_11937_amd as pz
    import workloads as wl
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    pz.lib()                                                      # fails loudly if libpz.so is not built
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
    ms_step_ev, kern_ms = time_steps(torch, layers, args.steps, args.warmup, events=True)
    attn_bytes = float(np.mean([l.attn_bytes(wl) for l in layers]))
    step_bytes = float(np.mean([l.step_bytes(wl) for l in layers]))
    B = spec["B"]
    kern_avg_ms = float(kern_ms.mean())
    result = {
        "metric": METRIC, "value": step_bytes / (ms_step * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "e4m3 KV -> bf16 MFMA operands, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": spec["text"], "batch": B, "n_q_heads": 64, "n_kv_heads": 8, "head_dim": 64,
                   "page_size": 64, "window": spec["window"], "split_tokens": spec["split_tokens"],
                   "cache_instances_rotated": len(layers)},
        "attn_tokens_per_s": B / (ms_step * 1e-3),
        "pct_hbm_peak": 100.0 * step_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "roofline": {"bound": "hbm", "kernel": "decode_attn_kernel<64,1>",
                     "achieved": attn_bytes / (kern_avg_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": attn_bytes / (kern_avg_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "kernel_us_avg": kern_avg_ms * 1e3, "kernel_us_std": float(kern_ms.std() * 1e3),
                     "ms_per_step_with_events": ms_step_ev,
                     "algorithmic_bytes_per_launch": attn_bytes,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(args.workload) if args.split_tokens is None else None},
    }
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
