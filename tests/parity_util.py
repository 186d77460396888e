"""Helpers for the GPU-vs-oracle parity tests: run the same seeded stream through the HIP
library (via its C ABI) and through the CPU oracle and compare every piece of state."""
from __future__ import annotations

import numpy as np

import synth_inputs as si
from oracle import xstream_oracle as xo

# Tolerances for the attention output, relative to unit-RMS outputs.
OUT_MAX_ABS = 2e-2
OUT_MEAN_ABS = 2e-3


def oracle_cfg(w: si.Workload, meta16: bool = False, slots: bool = False) -> xo.OracleConfig:
    return xo.OracleConfig(w.n_heads, w.head_dim, w.tokens_per_frame, w.n_special, w.pool_group, w.budget_tokens,
                           w.k_bits, w.k_group, w.v_bits, w.v_group, meta16=meta16, slot_stable=slots)


def make_handle(w: si.Workload, n_streams=1, n_layers=1, **extra):
    """Outputs are taken in fp32 so that the tolerance tests the arithmetic and not the
    8-bit significand of a bf16 store (half a bf16 ulp of an output ten times the RMS is
    already 2e-2 of the RMS); test_bf16_output_is_rounded_fp32_output covers the bf16 store."""
    import paper_2601_01204_amd as kvx
    extra.setdefault("out_dtype", kvx.KV_F32)
    return kvx.KvHandle(n_streams=n_streams, n_layers=n_layers, n_heads=w.n_heads, tokens_per_frame=w.tokens_per_frame,
                        n_special=w.n_special, pool_group=w.pool_group, budget_tokens=w.budget_tokens, k_bits=w.k_bits,
                        k_group=w.k_group, v_bits=w.v_bits, v_group=w.v_group,
                        in_dtype=kvx.KV_F32 if w.dtype == "f32" else kvx.KV_BF16, **extra)


def to_device(a: np.ndarray, w: si.Workload):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    return t if w.dtype == "f32" else t.to(torch.bfloat16)      # exact: values are bf16-representable


def check_output(got: np.ndarray, ref: np.ndarray, what: str):
    rms = float(np.sqrt((ref ** 2).mean()))
    err = np.abs(got.astype(np.float64) - ref) / rms
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    assert err.max() <= OUT_MAX_ABS, f"{what}: max abs err {err.max():.4g} (unit-RMS) > {OUT_MAX_ABS}"
    assert err.mean() <= OUT_MEAN_ABS, f"{what}: mean abs err {err.mean():.4g} (unit-RMS) > {OUT_MEAN_ABS}"
    return float(err.max()), float(err.mean())


def check_state(ex: dict, cache: xo.OracleCache, what: str):
    """Kept indices, codes and metadata are compared bit-for-bit."""
    assert ex["cache_len"] == cache.cache_len, f"{what}: cache_len {ex['cache_len']} != {cache.cache_len}"
    assert np.array_equal(ex["ids"], cache.ids), f"{what}: token ids differ"
    if cache.last_keep is not None:
        assert ex["last_keep"] is not None, f"{what}: no keep list exported"
        assert np.array_equal(ex["last_keep"], cache.last_keep), f"{what}: keep list differs"
        assert np.array_equal(ex["last_scores"].view(np.uint32), cache.last_scores.view(np.uint32)), f"{what}: scores differ in bits"
    else:
        assert ex["last_keep"] is None, f"{what}: unexpected keep list"
    for name, ref in (("k_scale", cache.Ks), ("v_scale", cache.Vs)):
        assert np.array_equal(ex[name].view(np.uint32), ref.view(np.uint32)), f"{what}: {name} differs in bits"
    for name, ref in (("k_zero", cache.Kz), ("v_zero", cache.Vz), ("k_codes", cache.Kc), ("v_codes", cache.Vc)):
        if not np.array_equal(ex[name], ref):
            bad = np.argwhere(ex[name] != ref)
            raise AssertionError(f"{what}: {name} differs at {len(bad)} places, first {bad[0].tolist()}: "
                                 f"{ex[name][tuple(bad[0])]} != {ref[tuple(bad[0])]}")


def run_stream(w: si.Workload, frames: int, check_every: int = 1, stream: int = 0, layer: int = 0, handle=None,
               log=print, meta16: bool = False, slots: bool = False):
    """Free-running parity: both sides evolve their own cache from the same inputs.  meta16: the
    16-bit quantiser metadata format on both sides; slots: the slot-stable layout on both sides."""
    import torch
    h = handle or make_handle(w, meta_format=1 if meta16 else 0, layout=1 if slots else 0)
    cache = xo.OracleCache(oracle_cfg(w, meta16, slots))
    sigma = si.key_channel_scales(w, stream, layer)
    worst = (0.0, 0.0)
    for t in range(frames):
        q, k, v = si.frame_qkv(w, t, stream, layer, sigma)
        ref = cache.step(q, k, v)
        tq, tk, tv = (to_device(a, w) for a in (q, k, v))
        out = torch.empty(tq.shape, dtype=torch.float32, device=tq.device)
        h.step(tq, tk, tv, out)
        torch.cuda.synchronize()
        e = check_output(out.float().cpu().numpy(), ref, f"{w.name} frame {t}")
        worst = (max(worst[0], e[0]), max(worst[1], e[1]))
        if t % check_every == 0 or t == frames - 1:
            check_state(h.export(), cache, f"{w.name} frame {t}")
        log(f"  {w.name} frame {t}: len {cache.cache_len} out err max {e[0]:.3g} mean {e[1]:.3g}", flush=True)
    if handle is None:
        h.close()
    return worst
