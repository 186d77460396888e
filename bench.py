#!/usr/bin/env python3
"""Benchmark of the compressed-KV streaming attention step on one MI355X.

A step is one kv_step() on the 'vggt_layer' workload (the benchmark's second configuration: one
VGGT-scale global-attention layer, 16 heads x 64, 1041 tokens per frame, budget 8192,
INT4 keys per channel / INT4 values per token, group 64) in steady state, i.e. with the
cache full so that every step attends over 8192 + 1041 keys, scores, prunes 1041 tokens
and re-quantises.  Inputs are synthetic and resident in HBM before the timed region.
Prints one JSON line.
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

PEAK_MFMA_TFLOPS = 2500.0      # MI355X dense bf16 / fp16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
# HBM bytes per attention launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (see
# profiles/attn_kernel_vggt_layer_counters.txt), fetch counter scaled by 2.00, write by 1.00.
ATTENTION_TRAFFIC_BYTES = 34.25e6


def oracle_baseline(w, frames_total=18, steady_from=9):
    """The CPU oracle as it stands, timed on this host: frames 0..frames_total-1 of the same
    stream; the rate is taken over the steady frames (cache full, pruning every step)."""
    import numpy as np
    import synth_inputs as si
    from oracle import xstream_oracle as xo
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    cfg = xo.OracleConfig(w.n_heads, w.head_dim, w.tokens_per_frame, w.n_special, w.pool_group, w.budget_tokens,
                          w.k_bits, w.k_group, w.v_bits, w.v_group)
    cache = xo.OracleCache(cfg)
    sigma = si.key_channel_scales(w)
    steady = []
    for t in range(frames_total):
        q, k, v = si.frame_qkv(w, t, sigma=sigma)
        t0 = time.perf_counter()
        cache.step(q, k, v)
        dt = time.perf_counter() - t0
        if t >= steady_from:
            steady.append(dt)
    return {"value": len(steady) / sum(steady), "unit": "frames/s", "cores": int(threads), "kind": "oracle",
            "sample": f"frames 0-{frames_total - 1} of the same stream run through the numpy oracle; rate over steady frames "
                      f"{steady_from}-{frames_total - 1} (cache full at {w.budget_tokens} tokens)"}


def aux_measurements(torch, kvx, si, dev, frames, peak_hbm):
    """Side measurements, outside the timed region of the headline number:
    (1) the attention kernel alone on the benchmark workload (no second stream, all CUs);
    (2) one batched step over the 24 independent layer caches of the 'vggt_stack' workload
        (budget 16384), which gives the bandwidth kernels launches large enough to be judged
        against HBM peak;
    (3) the uncompressed bf16 cache (plain Eq. 1 over every past frame) at 100, 250 and 500 frames
        of the benchmark workload: per-frame time and cache bytes grow with the stream, which is
        the growth the compressed cache's flat cost is set against (Sec. 4.3);
    (4) the matrix-instruction rate and the copy bandwidth this machine sustains."""
    out = {}
    w = si.WORKLOADS["vggt_layer"]
    n, H, d, L = w.tokens_per_frame, w.n_heads, w.head_dim, w.budget_tokens
    h = kvx.KvHandle(n_heads=H, tokens_per_frame=n, n_special=w.n_special, pool_group=w.pool_group, budget_tokens=L,
                     k_bits=w.k_bits, k_group=w.k_group, v_bits=w.v_bits, v_group=w.v_group)
    h.set_option("overlap_update", 0)
    o = torch.empty((n, H, d), dtype=torch.bfloat16, device=dev)
    for t in range(12):
        h.step(*frames[t % len(frames)], o)
    h.set_timing(1)
    for t in range(50):
        h.step(*frames[t % len(frames)], o)
    torch.cuda.synchronize()
    ms, cnt = h.read_timing()["attention"]
    us = ms * 1e3 / cnt
    out["attention_alone"] = {"us": round(us, 2), "TFLOP/s": round(4.0 * n * (L + n) * d * H / (us * 1e-6) / 1e12, 1)}
    h.close()

    w = si.WORKLOADS["vggt_stack"]
    n, H, d, L, NL = w.tokens_per_frame, w.n_heads, w.head_dim, w.budget_tokens, w.n_layers
    h = kvx.KvHandle(n_layers=NL, n_heads=H, tokens_per_frame=n, n_special=w.n_special, pool_group=w.pool_group,
                     budget_tokens=L, k_bits=w.k_bits, k_group=w.k_group, v_bits=w.v_bits, v_group=w.v_group)
    outs = [torch.empty((n, H, d), dtype=torch.bfloat16, device=dev) for _ in range(NL)]
    fill = -(-L // n) + 1

    def step(t):
        h.step_batched([(0, l, *frames[(t + l) % len(frames)], outs[l]) for l in range(NL)])
    for t in range(fill + 2):
        step(t)
    torch.cuda.synchronize()
    # throughput as deployed (cache update beside attention), then the kernels one after the other for their own times
    steps = 10
    t0 = time.perf_counter()
    for t in range(steps):
        step(fill + 2 + t)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    h.set_option("overlap_update", 0)
    h.set_timing(0x7F)
    for t in range(steps):
        step(fill + 2 + steps + t)
    torch.cuda.synchronize()
    tm = h.read_timing()
    kb, vb = w.k_bits, w.v_bits
    per_layer = {
        "score": H * L * d * kb / 8 + H * (L // w.k_group) * d * 8 + H * L * 4,
        "rebuild_k": 2 * (H * L * d * kb / 8 + H * (L // w.k_group) * d * 8) + n * H * d * 2,
        "rebuild_v": 2 * (H * L * d * vb / 8 + H * L * 8) + n * H * d * 2,
    }
    hb = {}
    for name, nbytes in per_layer.items():
        ms, cnt = tm[name]
        us = ms * 1e3 / cnt
        gbs = NL * nbytes / (us * 1e-6) / 1e9
        hb[name] = {"us": round(us, 2), "GB/s": round(gbs, 1), "frac": round(gbs / peak_hbm, 4)}
    # score and key rebuild are bound by vector-instruction issue, not memory: instructions per wave from
    # rocprofv3 SQ_INSTS_VALU / SQ_WAVES (profiles/update_kernels_vggt_stack_counters.txt, INT4 kernels), one wave
    # per 64 cached tokens and head (score) or per 16 tokens and head (rebuild), against the chip's issue rate of
    # one 64-lane instruction per SIMD every 4 cycles: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3 T lane-instr/s
    if kb == 4:
        peak_lane_instr = 256 * 4 * 16 * 2.4e9
        for name, per_wave, waves in (("score", 413.25, NL * H * (L // 64)), ("rebuild_k", 340.4, NL * H * (L // 16))):
            rate = per_wave * waves * 64 / (hb[name]["us"] * 1e-6)
            hb[name]["valu"] = {"bound": "alu", "achieved": round(rate / 1e12, 2), "peak": round(peak_lane_instr / 1e12, 2),
                                "unit": "T lane-instr/s", "frac": round(rate / peak_lane_instr, 4)}
    ms, cnt = tm["attention"]
    us = ms * 1e3 / cnt
    out["stack24_batched_step"] = {
        "frames/s (24-layer frames)": round(steps / dt, 2),
        "kernel_us": {k: round(v[0] * 1e3 / v[1], 2) for k, v in tm.items() if v[1]},
        "attention_TFLOP/s": round(NL * 4.0 * n * (L + n) * d * H / (us * 1e-6) / 1e12, 1),
        "hbm_kernels": hb,
        "kv_bytes_live_per_layer": h.stats()["bytes_live_per_cache"],
    }
    h.close()

    w = si.WORKLOADS["vggt_layer"]
    n, H, d = w.tokens_per_frame, w.n_heads, w.head_dim
    marks = (100, 250, 500)
    h = kvx.KvHandle(n_heads=H, tokens_per_frame=n, n_special=w.n_special, pool_group=w.pool_group,
                     budget_tokens=w.budget_tokens, mode=kvx.KV_UNCOMPRESSED_BF16, max_frames=marks[-1])
    o = torch.empty((n, H, d), dtype=torch.bfloat16, device=dev)
    growth = {}
    t = 0
    for m in marks:
        while t < m - 5:
            h.step(*frames[t % len(frames)], o)
            t += 1
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        while t < m:
            h.step(*frames[t % len(frames)], o)
            t += 1
        torch.cuda.synchronize()
        growth[str(m)] = {"ms_per_frame": round((time.perf_counter() - t0) * 1e3 / 5, 3),
                          "cache_bytes": 2 * H * m * n * d * 2}
    out["uncompressed_bf16_by_frames"] = growth
    h.close()

    # what this machine sustains: a register-resident bf16 MFMA loop on every CU (~5 ms per launch,
    # long enough for the clock to settle under the power limit) and a 1 GiB streaming copy
    out["machine"] = {"mfma_bf16_sustained_TFLOP/s": round(kvx.probe_mfma_bf16(50000, 3), 1),
                      "hbm_copy_GB/s": round(kvx.probe_copy(1 << 30, 3), 1)}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=24)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--splits", type=int, default=0, help="override the attention key-range split count")
    ap.add_argument("--no-overlap", action="store_true", help="run the cache update after attention instead of beside it")
    ap.add_argument("--no-aux", action="store_true", help="skip the auxiliary measurements (standalone attention, 24-layer batched step)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run 1 GiB device-to-device copies (copy_probe_kernel), the known-size reference for HBM byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2601_01204_amd as kvx
    import synth_inputs as si

    w = si.WORKLOADS["vggt_layer"]
    dev = torch.device("cuda:0")
    n, H, d, L = w.tokens_per_frame, w.n_heads, w.head_dim, w.budget_tokens
    h = kvx.KvHandle(n_heads=H, tokens_per_frame=n, n_special=w.n_special, pool_group=w.pool_group, budget_tokens=L,
                     k_bits=w.k_bits, k_group=w.k_group, v_bits=w.v_bits, v_group=w.v_group, in_dtype=kvx.KV_BF16,
                     out_dtype=kvx.KV_BF16)
    if args.splits:
        h.set_option("attention_splits", args.splits)
    if args.no_overlap:
        h.set_option("overlap_update", 0)

    if args.copy_calibration:
        kvx.probe_copy(1 << 30, 3)

    # a ring of distinct frames, resident in HBM
    ring = w.frames
    sigma = si.key_channel_scales(w)
    frames = []
    for t in range(ring):
        q, k, v = si.frame_qkv(w, t, sigma=sigma)
        frames.append(tuple(torch.from_numpy(a).to(dev).to(torch.bfloat16) for a in (q, k, v)))
    out = torch.empty((n, H, d), dtype=torch.bfloat16, device=dev)
    stream = torch.cuda.current_stream().cuda_stream

    fill = -(-L // n) + 1                       # frames until the cache is full and pruning every step
    warm = max(args.warmup, fill)
    t_idx = 0
    for _ in range(warm):
        q, k, v = frames[t_idx % ring]
        h.step(q, k, v, out, hip_stream=stream)
        t_idx += 1
    torch.cuda.synchronize()
    assert h.stats()["cache_len_max"] == L

    # HIP events around the attention kernel, on its stream, on every 8th step of the timed region: an event
    # pair costs the stream about 6 us, which would otherwise come out of every step of the headline figure
    h.set_option("timing_every", 8)
    h.set_timing(1 << 0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        q, k, v = frames[t_idx % ring]
        h.step(q, k, v, out, hip_stream=stream)
        t_idx += 1
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    attn_ms, attn_cnt = h.read_timing()["attention"]
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    assert bool(torch.isfinite(out.float()).all())

    # per-kernel durations of the whole step (separate pass: the extra events perturb the stream a little)
    h.set_option("timing_every", 1)
    h.set_timing(0x7F)
    for _ in range(min(args.steps, 50)):
        q, k, v = frames[t_idx % ring]
        h.step(q, k, v, out, hip_stream=stream)
        t_idx += 1
    torch.cuda.synchronize()
    per_kernel = h.read_timing()
    h.set_timing(0)
    st = h.stats()

    T = L + n
    flops = 4.0 * n * T * d * H
    attn_s = attn_ms * 1e-3 / max(attn_cnt, 1)
    achieved = flops / attn_s / 1e12
    kb, vb = w.k_bits, w.v_bits
    mid = L - n
    alg_bytes = {
        # middle key codes + their (s, z) + the D[h, j] written
        "score": H * L * d * kb / 8 + H * (L // w.k_group) * d * 8 + H * L * 4,
        # survivors' key codes + (s, z) read, new frame read, next cache written
        "rebuild_k": 2 * (H * L * d * kb / 8 + H * (L // w.k_group) * d * 8) + n * H * d * 2,
        "rebuild_v": 2 * (H * L * d * vb / 8 + H * L * 8) + n * H * d * 2,
        "select": H * mid * 4 + 6 * mid * 4 + L * 4,
    }
    hbm = {}
    for name, nbytes in alg_bytes.items():
        ms, cnt = per_kernel[name]
        if cnt:
            us = ms * 1e3 / cnt
            hbm[name] = {"us": round(us, 2), "GB/s": round(nbytes / (us * 1e-6) / 1e9, 1), "frac": round(nbytes / (us * 1e-6) / 1e9 / PEAK_HBM_GBS, 4)}
    kernels_us = {k: round(v[0] * 1e3 / v[1], 2) for k, v in per_kernel.items() if v[1]}

    res = {
        "metric": "frames/s of compressed-KV causal attention step",
        "value": round(args.steps / (t1 - t0), 2),
        "unit": "frames/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": warm,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "vggt_layer: 1 layer, 16 heads x 64, 1041 tokens/frame, budget 8192, INT4 K per-channel g64 / INT4 V per-token g64, steady state",
                   "keys_per_step": T, "attention_splits": args.splits or "auto"},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK_MFMA_TFLOPS, 4), "traffic": ATTENTION_TRAFFIC_BYTES,
                     "kernel": "attn_kernel", "flops_per_launch": flops, "avg_launch_us": round(attn_s * 1e6, 2)},
        "hbm_kernels": hbm,
        "kernel_us": kernels_us,
        "kv_bytes": {"live_per_cache": st["bytes_live_per_cache"], "allocated": st["bytes_allocated"],
                     "bf16_uncompressed_equivalent": 2 * H * L * d * 2},
    }
    h.close()

    if not args.no_aux:
        res["aux"] = aux_measurements(torch, kvx, si, dev, frames, PEAK_HBM_GBS)
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = oracle_baseline(w)
    else:
        res["cpu_baseline"] = None
    print(json.dumps(res))


if __name__ == "__main__":
    main()
