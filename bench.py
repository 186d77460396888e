#!/usr/bin/env python3
"""Benchmark of the compressed-KV streaming attention step on one MI355X.

A step is one frame of the 'vggt_stack' workload (the benchmark's third configuration, the one
its work figures are quoted on): 24 independent per-layer caches of a VGGT-scale global-attention
stack, 16 heads x 64, 1041 tokens per frame, budget 16384 tokens per layer, INT4 keys per channel /
INT4 values per token, group 64, stepped by one kv_step_batched() call, in steady state (every cache
full, so every layer attends over 16384 + 1041 keys, scores, prunes 1041 tokens and re-quantises).
Inputs are synthetic, generated on the device and resident in HBM before the timed region.
Prints one JSON line.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_TFLOPS = 2500.0      # MI355X dense bf16 / fp16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
# HBM bytes per launch of the dominant kernel come from a rocprofv3 --pmc run whose summary and figures are
# tracked in profiles/; the file names the sources it was measured on, and a stale file yields traffic = null.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "attn_kernel_vggt_stack_traffic.json")
KERNEL_SOURCES = ("attn.hip", "attn16.hip", "kvx_dev.h")


def kernel_source_hash() -> str:
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2601_01204_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def attention_traffic(workload: str, meta: str):
    """HBM bytes per attention launch as the counters measured them, or None when the tracked figure
    was taken on other sources or another workload."""
    try:
        with open(TRAFFIC_FILE) as f:
            t = json.load(f)
    except (OSError, ValueError):
        return None
    if t.get("workload") != workload or t.get("metadata") != meta or t.get("source_sha256_16") != kernel_source_hash():
        return None
    return float(t["hbm_bytes_per_launch"])


def device_frames(torch, w, dev, caches, ring, seed):
    """ring distinct frames per cache, generated on the device: Q, V ~ N(0, 1), K ~ N(0, 1) times a
    per-(cache, head, channel) log-normal scale, rounded to bf16 (the recipe of synth_inputs, drawn by
    torch's device generator so that 24-96 caches x 20 frames need no host time)."""
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    n, H, d = w.tokens_per_frame, w.n_heads, w.head_dim
    out = []
    for _ in range(caches):
        sigma = torch.exp(torch.randn((H, d), generator=gen, device=dev))
        q = torch.randn((ring, n, H, d), generator=gen, device=dev).to(torch.bfloat16)
        k = (torch.randn((ring, n, H, d), generator=gen, device=dev) * sigma).to(torch.bfloat16)
        v = torch.randn((ring, n, H, d), generator=gen, device=dev).to(torch.bfloat16)
        out.append((q, k, v))
    return out


def alg_bytes(w, meta_bytes=8):
    """Algorithmic HBM bytes of the bandwidth kernels per cache-step in steady state (cache full)."""
    n, H, d, L = w.tokens_per_frame, w.n_heads, w.head_dim, w.budget_tokens
    kb, vb = w.k_bits, w.v_bits
    mid = L - n
    k_meta = H * (L // w.k_group) * d * meta_bytes
    v_meta = H * L * (d // w.v_group) * meta_bytes
    return {
        # middle key codes + their (s, z) read, D[h, j] written
        "score": H * mid * d * kb / 8 + H * (mid // w.k_group) * d * meta_bytes + H * mid * 4,
        # survivors' key codes + (s, z) read, new frame read, next cache written
        "rebuild_k": 2 * (H * L * d * kb / 8 + k_meta) + n * H * d * 2,
        "rebuild_v": 2 * (H * L * d * vb / 8 + v_meta) + n * H * d * 2,
        "select": H * mid * 4 + 6 * mid * 4 + L * 4,
    }


def attention_flops(w):
    n, H, d, L = w.tokens_per_frame, w.n_heads, w.head_dim, w.budget_tokens
    return 4.0 * n * (L + n) * d * H


class StackRun:
    """caches = n_streams x n_layers caches of workload w, all stepped by one kv_step_batched per frame."""

    def __init__(self, torch, kvx, w, dev, n_streams, n_layers, ring, seed, **extra):
        self.torch, self.w = torch, w
        self.n_streams, self.n_layers = n_streams, n_layers
        self.h = kvx.KvHandle(n_streams=n_streams, n_layers=n_layers, n_heads=w.n_heads, tokens_per_frame=w.tokens_per_frame,
                              n_special=w.n_special, pool_group=w.pool_group, budget_tokens=w.budget_tokens, k_bits=w.k_bits,
                              k_group=w.k_group, v_bits=w.v_bits, v_group=w.v_group, in_dtype=kvx.KV_BF16,
                              out_dtype=kvx.KV_BF16, **extra)
        nc = n_streams * n_layers
        self.frames = device_frames(torch, w, dev, nc, ring, seed)
        self.ring = ring
        self.outs = [torch.empty((w.tokens_per_frame, w.n_heads, w.head_dim), dtype=torch.bfloat16, device=dev) for _ in range(nc)]
        self.t = 0
        self.stream = torch.cuda.current_stream().cuda_stream

    def step(self):
        r = self.t % self.ring
        items = []
        for s in range(self.n_streams):
            for l in range(self.n_layers):
                c = s * self.n_layers + l
                q, k, v = self.frames[c]
                items.append((s, l, q[r], k[r], v[r], self.outs[c]))
        self.h.step_batched(items, hip_stream=self.stream)
        self.t += 1

    def run(self, steps):
        for _ in range(steps):
            self.step()

    def timed(self, steps):
        self.torch.cuda.synchronize()
        t0 = time.perf_counter()
        self.run(steps)
        self.torch.cuda.synchronize()
        return time.perf_counter() - t0

    def close(self):
        self.h.close()


def kernel_times(run, steps):
    """Per-kernel durations with the cache update after attention on one stream (each kernel by itself)."""
    run.h.set_option("overlap_update", 0)
    run.h.set_option("timing_every", 1)
    run.h.set_timing(0x7F)
    run.run(steps)
    run.torch.cuda.synchronize()
    tm = run.h.read_timing()
    run.h.set_timing(0)
    run.h.set_option("overlap_update", 1)
    return {k: v[0] * 1e3 / v[1] for k, v in tm.items() if v[1]}


def hbm_report(w, n_caches_per_launch, us, meta_bytes=8):
    out = {}
    for name, nbytes in alg_bytes(w, meta_bytes).items():
        if name in us:
            gbs = n_caches_per_launch * nbytes / (us[name] * 1e-6) / 1e9
            out[name] = {"us": round(us[name], 2), "bytes": int(n_caches_per_launch * nbytes), "GB/s": round(gbs, 1),
                         "frac": round(gbs / PEAK_HBM_GBS, 4)}
    return out


def oracle_baseline(torch, run, frames_total, steady, meta16=False):
    """The CPU oracle as it stands, timed on this host on one layer cache of the same stream (the frames the GPU's
    layer 0 was fed, copied back): frames 0..frames_total-1, the last `steady` of them with the cache full.  The
    24-layer rate is one over 24 times the steady per-layer step time (the oracle's layers are independent)."""
    import numpy as np
    from oracle import xstream_oracle as xo
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    w = run.w
    cfg = xo.OracleConfig(w.n_heads, w.head_dim, w.tokens_per_frame, w.n_special, w.pool_group, w.budget_tokens,
                          w.k_bits, w.k_group, w.v_bits, w.v_group, meta16=meta16)
    cache = xo.OracleCache(cfg)
    q, k, v = run.frames[0]
    times = []
    for t in range(frames_total):
        r = t % run.ring
        fq, fk, fv = (a[r].float().cpu().numpy() for a in (q, k, v))
        t0 = time.perf_counter()
        cache.step(fq, fk, fv)
        times.append(time.perf_counter() - t0)
    per_layer = sum(times[-steady:]) / steady
    return {"value": 1.0 / (run.n_layers * per_layer), "unit": "frames/s", "cores": int(threads), "kind": "oracle",
            "sample": f"layer 0 of the same stream through the numpy oracle, frames 0-{frames_total - 1} ({sum(times):.1f} s of CPU "
                      f"work); steady per-layer step {per_layer * 1e3:.0f} ms over the last {steady} frames (cache full at "
                      f"{w.budget_tokens} tokens), times {run.n_layers} layers"}


def stack_variant(torch, kvx, w, dev, NL, warm, steps, meta16, slots, flops):
    """The headline 24-layer step with another metadata format and / or cache layout."""
    run2 = StackRun(torch, kvx, w, dev, 1, NL, 20, 102, meta_format=kvx.KV_META_F16 if meta16 else kvx.KV_META_F32,
                    layout=kvx.KV_LAYOUT_SLOTS if slots else kvx.KV_LAYOUT_COMPACT)
    run2.run(warm)
    run2.h.set_option("timing_every", 1)
    run2.h.set_timing(1)
    dt2 = run2.timed(steps)
    ms2, cnt2 = run2.h.read_timing()["attention"]
    run2.h.set_timing(0)
    us2 = kernel_times(run2, min(steps, 10))
    st2 = run2.h.stats()
    a2 = ms2 * 1e-3 / max(cnt2, 1)
    out = {"workload": "the headline step with " + ("16-bit scale + zero-point" if meta16 else "fp32 scale + int32 zero-point") +
                       " metadata, " + ("slot-stable" if slots else "compacting") + " layout",
           "frames/s": round(steps / dt2, 2), "ms_per_step": round(dt2 * 1e3 / steps, 4),
           "attention_us": round(a2 * 1e6, 2), "attention_TFLOP/s": round(flops / a2 / 1e12, 1),
           "attention_frac": round(flops / a2 / 1e12 / PEAK_MFMA_TFLOPS, 4),
           "kernel_us": {k: round(v, 2) for k, v in us2.items()},
           "kv_bytes": {"live_per_cache": st2["bytes_live_per_cache"], "allocated": st2["bytes_allocated"],
                        "allocated_per_cache": st2["bytes_allocated"] // NL}}
    if not slots:
        out["hbm_kernels"] = hbm_report(w, NL, us2, 4 if meta16 else 8)
    run2.close()
    return out


def aux_vggt_layer(torch, kvx, si, dev, steps):
    """One layer cache of the second configuration (budget 8192) through kv_step: the latency a model whose
    layers run one after the other sees per layer; the same with 16-bit metadata, with four frames per call
    (kv_step_frames, frame-wise causal mask inside the chunk) and in the update-first order."""
    w = si.WORKLOADS["vggt_layer"]
    n, H, d = w.tokens_per_frame, w.n_heads, w.head_dim
    fill = -(-w.budget_tokens // n) + 1
    out = {"workload": "vggt_layer: 1 layer, budget 8192, INT4/INT4 g64, one cache per call"}
    variants = (("kv_step", dict(), 1), ("kv_step_meta16", dict(meta_format=kvx.KV_META_F16), 1),
                ("kv_step_frames_4", dict(max_frames_per_step=4), 4),
                ("kv_step_frames_4_meta16", dict(max_frames_per_step=4, meta_format=kvx.KV_META_F16), 4),
                ("kv_step_update_first", dict(order=kvx.KV_PRUNE_THEN_ATTEND), 1))
    for name, extra, F in variants:
        run = StackRun(torch, kvx, w, dev, 1, 1, 12, 101, **extra)
        q, k, v = run.frames[0]
        o = torch.empty((F * n, H, d), dtype=torch.bfloat16, device=dev)

        def call(i):
            r = (i * F) % 12
            run.h.step_frames(F, q[r:r + F].reshape(F * n, H, d), k[r:r + F].reshape(F * n, H, d), v[r:r + F].reshape(F * n, H, d),
                              o, hip_stream=run.stream)
        calls = max(steps // F, 10)
        for i in range(fill + 3):
            call(i)
        run.h.set_option("timing_every", 8 if F == 1 else 1)
        run.h.set_timing(1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(calls):
            call(i)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        ms, cnt = run.h.read_timing()["attention"]
        run.h.set_timing(0)
        a_us = ms * 1e3 / max(cnt, 1)
        # attention flops of a call: every frame's queries over the cache and the chunk's frames up to their own
        flops = sum(4.0 * n * (w.budget_tokens + (f + 1) * n) * d * H for f in range(F))
        if name == "kv_step_update_first":
            flops = 4.0 * n * w.budget_tokens * d * H
        st = run.h.stats()
        out[name] = {"frames/s": round(F * calls / dt, 1), "ms_per_call": round(dt * 1e3 / calls, 4), "attention_us": round(a_us, 2),
                     "attention_TFLOP/s": round(flops / (a_us * 1e-6) / 1e12, 1),
                     "attention_frac": round(flops / (a_us * 1e-6) / 1e12 / PEAK_MFMA_TFLOPS, 4),
                     "kv_bytes": {"live_per_cache": st["bytes_live_per_cache"], "allocated": st["bytes_allocated"]}}
        if name == "kv_step":
            out[name]["kernel_us"] = {kk: round(vv, 2) for kk, vv in kernel_times(run, min(steps, 50)).items()}
        run.close()
    return out


def aux_small_budgets(torch, kvx, si, dev, steps):
    """The paper's own cache budgets (L_max = 2K in its experiments, 2K-8K in its ablation) on one layer cache:
    the step is then bound by the launch latencies of the update chain rather than by any roofline.  L = 2048
    needs frames of at most 1024 tokens (first and current frame are always kept), so it runs on 518 x 294 frames
    (782 tokens); 4096 and 8192 on 518 x 392 frames (1041 tokens)."""
    import dataclasses
    out = {}
    base = si.WORKLOADS["vggt_layer"]
    for n, L in ((782, 2048), (1041, 4096), (1041, 8192)):
        w = dataclasses.replace(base, tokens_per_frame=n, budget_tokens=L)
        for meta16 in (False, True):
            run = StackRun(torch, kvx, w, dev, 1, 1, 12, 107, meta_format=kvx.KV_META_F16 if meta16 else kvx.KV_META_F32)
            run.run(-(-L // n) + 3)
            dt = run.timed(steps)
            us = kernel_times(run, min(steps, 50))
            out[f"n{n}_L{L}_meta_{'f16' if meta16 else 'f32'}"] = {
                "frames/s": round(steps / dt, 1), "us_per_step": round(dt * 1e6 / steps, 1),
                "kernel_us": {k: round(v, 2) for k, v in us.items()}}
            run.close()
    return out


def aux_vggt_long(torch, kvx, si, dev, frames_total, unc_marks, meta16):
    """Fourth configuration: 24 layers streamed for frames_total frames with the compressed cache (per-frame time
    and allocated bytes sampled along the way), against the uncompressed bf16 cache of the same 24 layers at the
    marks in unc_marks (plain Eq. 1 over every past frame)."""
    w = si.WORKLOADS["vggt_long"]
    out = {"workload": f"vggt_long: 24 layers x {frames_total} frames, budget 16384, INT4/INT4 g64, " +
           ("16-bit" if meta16 else "fp32 + int32") + " metadata"}
    run = StackRun(torch, kvx, w, dev, 1, w.n_layers, 20, 103, meta_format=kvx.KV_META_F16 if meta16 else kvx.KV_META_F32)
    marks = sorted({m for m in (1, 100, 250, 500, 1000) if m <= frames_total} | {frames_total})
    comp = {}
    for m in marks:
        span = min(10, m - run.t)
        run.run(m - span - run.t)
        dt = run.timed(span)
        st = run.h.stats()
        comp[str(m)] = {"ms_per_frame": round(dt * 1e3 / span, 3), "cache_len": st["cache_len_max"],
                        "bytes_allocated": st["bytes_allocated"], "bytes_live": st["bytes_live_per_cache"] * w.n_layers}
    out["compressed_by_frames"] = comp
    frames_c = run.frames
    run.close()
    unc = {}
    last = max(unc_marks)
    h = kvx.KvHandle(n_layers=w.n_layers, n_heads=w.n_heads, tokens_per_frame=w.tokens_per_frame, n_special=w.n_special,
                     pool_group=w.pool_group, budget_tokens=w.budget_tokens, mode=kvx.KV_UNCOMPRESSED_BF16, max_frames=last)
    outs = [torch.empty((w.tokens_per_frame, w.n_heads, w.head_dim), dtype=torch.bfloat16, device=dev) for _ in range(w.n_layers)]
    t = 0

    def step():
        nonlocal t
        r = t % 20
        h.step_batched([(0, l, frames_c[l][0][r], frames_c[l][1][r], frames_c[l][2][r], outs[l]) for l in range(w.n_layers)])
        t += 1
    for m in sorted(unc_marks):
        while t < m - 3:
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        while t < m:
            step()
        torch.cuda.synchronize()
        unc[str(m)] = {"ms_per_frame": round((time.perf_counter() - t0) * 1e3 / 3, 2),
                       "cache_bytes": 2 * w.n_layers * w.n_heads * m * w.tokens_per_frame * w.head_dim * 2,
                       "bytes_allocated": h.stats()["bytes_allocated"]}
    h.close()
    out["uncompressed_bf16_by_frames"] = unc
    return out


def aux_vggt_hires(torch, kvx, si, dev, steps, meta16):
    """Fifth configuration: 4 streams x 24 layers, 1374 tokens per frame, budget 24576, INT2 keys g32 / INT4 values."""
    w = si.WORKLOADS["vggt_hires"]
    run = StackRun(torch, kvx, w, dev, w.n_streams, w.n_layers, 20, 105, meta_format=kvx.KV_META_F16 if meta16 else kvx.KV_META_F32)
    fill = -(-w.budget_tokens // w.tokens_per_frame) + 1
    run.run(fill + 2)
    dt = run.timed(steps)
    us = kernel_times(run, min(steps, 10))
    st = run.h.stats()
    launches = 2          # 96 caches = two launches of 48
    per_launch = w.n_streams * w.n_layers / launches
    out = {"workload": "vggt_hires: 4 streams x 24 layers in one kv_step_batched, 1374 tokens/frame, budget 24576, INT2 K g32 / INT4 V g64, " +
                       ("16-bit" if meta16 else "fp32 + int32") + " metadata",
           "frames/s (4-stream x 24-layer frames)": round(steps / dt, 2), "ms_per_step": round(dt * 1e3 / steps, 3),
           "stream_frames/s": round(w.n_streams * steps / dt, 2),
           "attention_TFLOP/s": round(per_launch * attention_flops(w) / (us["attention"] * 1e-6) / 1e12, 1),
           "attention_frac": round(per_launch * attention_flops(w) / (us["attention"] * 1e-6) / 1e12 / PEAK_MFMA_TFLOPS, 4),
           "kernel_us_per_launch_of_48": {k: round(v, 2) for k, v in us.items()},
           "hbm_kernels": hbm_report(w, per_launch, us, 4 if meta16 else 8),
           "kv_bytes": {"live_per_cache": st["bytes_live_per_cache"], "allocated": st["bytes_allocated"]}}
    run.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--splits", type=int, default=0, help="override the attention key-range split count")
    ap.add_argument("--no-overlap", action="store_true", help="run the cache update after attention instead of beside it")
    ap.add_argument("--overlap", type=int, default=None, choices=(0, 1, 2),
                    help="the library's overlap_update option: 0 in order, 1 the library's choice (default), 2 always beside")
    ap.add_argument("--no-aux", action="store_true", help="skip the other configurations (one layer, long stream, high-resolution multi-stream)")
    ap.add_argument("--long-frames", type=int, default=1000, help="frames of the long-stream run in aux")
    ap.add_argument("--layout", choices=("compact", "slots"), default="compact",
                    help="cache layout of the headline run: compacting double buffer, or slot-stable single buffer")
    ap.add_argument("--meta", choices=("f32", "f16"), default="f16",
                    help="quantiser metadata format of the headline run: fp32 scale + int32 zero-point, or 16-bit scale + zero-point")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run 1 GiB device-to-device copies (copy_probe_kernel), the known-size reference for HBM byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2601_01204_amd as kvx
    import synth_inputs as si

    dev = torch.device("cuda:0")
    if args.copy_calibration:
        kvx.probe_copy(1 << 30, 3)

    w = si.WORKLOADS["vggt_stack"]
    n, H, d, L, NL = w.tokens_per_frame, w.n_heads, w.head_dim, w.budget_tokens, w.n_layers
    meta16 = args.meta == "f16"
    slots = args.layout == "slots"
    run = StackRun(torch, kvx, w, dev, 1, NL, 20, 102, meta_format=kvx.KV_META_F16 if meta16 else kvx.KV_META_F32,
                   layout=kvx.KV_LAYOUT_SLOTS if slots else kvx.KV_LAYOUT_COMPACT)
    if args.splits:
        run.h.set_option("attention_splits", args.splits)
    if args.no_overlap:
        run.h.set_option("overlap_update", 0)
    elif args.overlap is not None:
        run.h.set_option("overlap_update", args.overlap)
    fill = -(-L // n) + 1                       # frames until every cache is full and prunes every step
    warm = max(args.warmup, fill)
    run.run(warm)
    torch.cuda.synchronize()
    assert run.h.stats()["cache_len_min"] == L

    # HIP events around the attention kernel on its own stream, inside the timed region (a pair costs the stream
    # a few microseconds of a 3 ms step)
    run.h.set_option("timing_every", 1)
    run.h.set_timing(1 << 0)
    dt = run.timed(args.steps)
    attn_ms, attn_cnt = run.h.read_timing()["attention"]
    run.h.set_timing(0)
    assert all(bool(torch.isfinite(o.float()).all()) for o in run.outs)
    us = kernel_times(run, min(args.steps, 20))
    st = run.h.stats()

    flops = NL * attention_flops(w)
    attn_s = attn_ms * 1e-3 / max(attn_cnt, 1)
    achieved = flops / attn_s / 1e12
    res = {
        "metric": "frames/s of compressed-KV causal attention step",
        "value": round(args.steps / dt, 2),
        "unit": "frames/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": warm,
        "ms_per_step": round(dt * 1e3 / args.steps, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "vggt_stack: 24 layer caches per frame in one kv_step_batched, 16 heads x 64, 1041 tokens/frame, budget "
                               "16384 tokens/layer, INT4 K per-channel g64 / INT4 V per-token g64, " +
                               ("16-bit scale + zero-point" if meta16 else "fp32 scale + int32 zero-point") +
                               (", slot-stable layout" if slots else ", compacting layout") + ", steady state",
                   "keys_per_step": L + n, "layers": NL, "attention_splits": args.splits or "auto"},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK_MFMA_TFLOPS, 4), "traffic": attention_traffic("vggt_stack", args.meta),
                     "kernel": "attn16_kernel" if meta16 else "attn_kernel", "flops_per_launch": flops, "avg_launch_us": round(attn_s * 1e6, 2)},
        "hbm_kernels": hbm_report(w, NL, us, 4 if meta16 else 8),
        "kernel_us": {k: round(v, 2) for k, v in us.items()},
        "kv_bytes": {"live_per_cache": st["bytes_live_per_cache"], "live_per_frame_step": st["bytes_live_per_cache"] * NL,
                     "allocated": st["bytes_allocated"], "allocated_per_cache": st["bytes_allocated"] // NL,
                     "bf16_uncompressed_equivalent_per_cache": 2 * H * L * d * 2,
                     "allocated_over_bf16_equivalent": round(st["bytes_allocated"] / NL / (2 * H * L * d * 2), 3)},
    }
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = oracle_baseline(torch, run, fill + 3, 3, meta16)
    else:
        res["cpu_baseline"] = None
    run.close()

    if not args.no_aux:
        aux = {}
        # the same 24-layer step in the other quantiser metadata format and in the other layout
        variants = [("meta_" + ("f32" if meta16 else "f16"), not meta16, slots), ("layout_" + ("compact" if slots else "slots"), meta16, not slots)]
        for vname, v_meta16, v_slots in variants:
            aux["vggt_stack_" + vname] = stack_variant(torch, kvx, w, dev, NL, warm, min(args.steps, 30), v_meta16, v_slots, flops)
        aux["vggt_layer"] = aux_vggt_layer(torch, kvx, si, dev, max(args.steps, 50))
        aux["small_budgets"] = aux_small_budgets(torch, kvx, si, dev, max(args.steps, 100))
        aux["vggt_long"] = aux_vggt_long(torch, kvx, si, dev, args.long_frames, (100, 250, 500), meta16)
        aux["vggt_hires"] = aux_vggt_hires(torch, kvx, si, dev, min(args.steps, 20), meta16)
        # what this machine sustains: a register-resident bf16 MFMA loop on every CU (~5 ms per launch,
        # long enough for the clock to settle under the power limit) and a 1 GiB streaming copy
        aux["machine"] = {"mfma_bf16_sustained_TFLOP/s": round(kvx.probe_mfma_bf16(50000, 3), 1),
                          "hbm_copy_GB/s": round(kvx.probe_copy(1 << 30, 3), 1)}
        res["aux"] = aux
    print(json.dumps(res))


if __name__ == "__main__":
    main()
