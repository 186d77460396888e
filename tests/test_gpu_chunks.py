"""GPU parity for calls that carry a chunk of frames (kv_step_frames: the frame-wise causal mask of Sec. 3.1 Eq. 1
inside the chunk, the chunk appended as one block of current tokens) and for the update-first order
(KV_PRUNE_THEN_ATTEND), against the oracle's variants.  Same bars as the single-frame tests: kept indices, scores,
codes, scales and zero-points bit-exact; outputs max abs <= 2e-2 and mean abs <= 2e-3 of unit-RMS."""
import dataclasses

import numpy as np
import pytest

import synth_inputs as si
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _run_chunked(w, chunks, meta16=False, f_max=None, **handle_extra):
    import torch
    from oracle import xstream_oracle as xo
    f_max = f_max or max(chunks)
    h = pu.make_handle(w, meta_format=1 if meta16 else 0, max_frames_per_step=f_max, **handle_extra)
    cache = xo.OracleCache(pu.oracle_cfg(w, meta16))
    sigma = si.key_channel_scales(w)
    t = 0
    for ci, F in enumerate(chunks):
        fr = [si.frame_qkv(w, t + f, sigma=sigma) for f in range(F)]
        q, k, v = (np.concatenate([f[j] for f in fr], axis=0) for j in range(3))
        ref = cache.step(q, k, v)
        tq, tk, tv = (pu.to_device(a, w) for a in (q, k, v))
        out = torch.full(tq.shape, float("nan"), dtype=torch.float32, device=tq.device)
        h.step_frames(F, tq, tk, tv, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        e = pu.check_output(got, ref, f"{w.name} call {ci} ({F} frames from {t})")
        for f in range(F):       # every frame of the chunk by itself, so that a small frame error cannot hide in the chunk's mean
            n = w.tokens_per_frame
            pu.check_output(got[f * n:(f + 1) * n], ref[f * n:(f + 1) * n], f"{w.name} call {ci} frame {t + f}")
        pu.check_state(h.export(), cache, f"{w.name} call {ci}")
        print(f"  {w.name} call {ci}: {F} frames, len {cache.cache_len}, err {e}", flush=True)
        t += F
    st = h.stats()
    assert st["frames_seen_total"] == t
    h.close()


@pytest.mark.parametrize("meta16", [False, True])
@pytest.mark.parametrize("k_bits,k_group,v_bits,v_group", [(4, 64, 4, 64), (2, 32, 4, 32)])
def test_small_chunks_of_mixed_length(meta16, k_bits, k_group, v_bits, v_group):
    """n = 70, budget 500: calls of 1, 2 and 3 frames in turn; the mask cuts through 64-key tiles, and the own keys
    of a 3-frame chunk span four tiles of which the early frames' queries skip the last ones."""
    w = si.Workload("chunks", 3, 64, 70, 5, 16, 500, 0, 1, 1, k_bits, k_group, v_bits, v_group, "bf16", 61)
    _run_chunked(w, [2, 1, 3, 3, 2, 1, 3], meta16=meta16)


def test_chunks_with_fp32_inputs_and_explicit_splits():
    w = si.Workload("chunks32", 2, 64, 133, 5, 16, 700, 0, 1, 1, 8, 64, 8, 64, "f32", 62)
    import torch
    from oracle import xstream_oracle as xo
    for splits in (1, 5):
        h = pu.make_handle(w, max_frames_per_step=4)
        h.set_option("attention_splits", splits)
        cache = xo.OracleCache(pu.oracle_cfg(w))
        sigma = si.key_channel_scales(w)
        t = 0
        for F in (4, 1, 2, 4):
            fr = [si.frame_qkv(w, t + f, sigma=sigma) for f in range(F)]
            q, k, v = (np.concatenate([f[j] for f in fr], axis=0) for j in range(3))
            ref = cache.step(q, k, v)
            tq, tk, tv = (pu.to_device(a, w) for a in (q, k, v))
            out = torch.empty(tq.shape, dtype=torch.float32, device=tq.device)
            h.step_frames(F, tq, tk, tv, out)
            torch.cuda.synchronize()
            pu.check_output(out.cpu().numpy(), ref, f"chunks32 splits {splits} frames {t}..")
            pu.check_state(h.export(), cache, f"chunks32 splits {splits} frames {t}..")
            t += F
        h.close()


@pytest.mark.parametrize("meta16", [False, True])
def test_vggt_layer_two_frames_per_call(meta16):
    """1041 tokens x 16 heads, budget 8192, two frames per call: six calls, pruning from the fourth (8 x 1041 > 8192)."""
    _run_chunked(si.WORKLOADS["vggt_layer"], [2] * 6, meta16=meta16)


def test_uncompressed_cache_takes_chunks():
    """The bf16 baseline cache with three frames per call equals plain Eq. 1 with the frame-wise causal mask."""
    import torch
    import paper_2601_01204_amd as kvx
    from oracle import xstream_oracle as xo
    w = si.Workload("unc_chunks", 2, 64, 133, 5, 16, 500, 0, 1, 1, 4, 64, 4, 64, "bf16", 63)
    h = pu.make_handle(w, mode=kvx.KV_UNCOMPRESSED_BF16, max_frames=7, max_frames_per_step=3)
    sigma = si.key_channel_scales(w)
    frames = [si.frame_qkv(w, t, sigma=sigma) for t in range(7)]
    t = 0
    for F in (3, 1, 3):
        q, k, v = (np.concatenate([f[j] for f in frames[t:t + F]], axis=0) for j in range(3))
        tq, tk, tv = (pu.to_device(a, w) for a in (q, k, v))
        out = torch.empty(tq.shape, dtype=torch.float32, device=tq.device)
        h.step_frames(F, tq, tk, tv, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        n = w.tokens_per_frame
        for f in range(F):
            ref = xo.reference_full_attention(frames, t + f, 1.0 / 8.0)
            pu.check_output(got[f * n:(f + 1) * n], ref, f"uncompressed frame {t + f}")
        t += F
    with pytest.raises(kvx.KvError) as e:          # one more frame would exceed max_frames
        h.step_frames(1, tq[:n], tk[:n], tv[:n], out[:n])
    assert e.value.code == -4
    h.close()


def test_chunk_length_is_validated():
    import torch
    import paper_2601_01204_amd as kvx
    w = si.Workload("chunk_err", 2, 64, 70, 5, 16, 300, 0, 1, 1, 4, 64, 4, 64, "bf16", 64)
    h = pu.make_handle(w, max_frames_per_step=2)
    x = torch.zeros((3 * 70, 2, 64), dtype=torch.bfloat16, device="cuda:0")
    o = torch.zeros(x.shape, dtype=torch.float32, device="cuda:0")
    for bad in (0, 3):
        with pytest.raises(kvx.KvError) as e:
            h.step_frames(bad, x, x, x, o)
        assert e.value.code == -3
    assert h.stats()["frames_seen_total"] == 0
    h.close()


# ----------------------------------------------------------------------------- update first, then attend
def _run_update_first(w, frames, meta16):
    import torch
    import paper_2601_01204_amd as kvx
    from oracle import xstream_oracle as xo
    h = pu.make_handle(w, meta_format=1 if meta16 else 0, order=kvx.KV_PRUNE_THEN_ATTEND)
    cfg = dataclasses.replace(pu.oracle_cfg(w, meta16), attend_after_prune=True)
    cache = xo.OracleCache(cfg)
    sigma = si.key_channel_scales(w)
    for t in range(frames):
        q, k, v = si.frame_qkv(w, t, sigma=sigma)
        ref = cache.step(q, k, v)
        tq, tk, tv = (pu.to_device(a, w) for a in (q, k, v))
        out = torch.full(tq.shape, float("nan"), dtype=torch.float32, device=tq.device)
        h.step(tq, tk, tv, out)
        torch.cuda.synchronize()
        e = pu.check_output(out.cpu().numpy(), ref, f"{w.name} update-first frame {t}")
        pu.check_state(h.export(), cache, f"{w.name} update-first frame {t}")
        print(f"  {w.name} update-first frame {t}: len {cache.cache_len} err {e}", flush=True)
    h.close()


@pytest.mark.parametrize("meta16", [False, True])
def test_update_first_order_small(meta16):
    w = si.Workload("upd_first", 3, 64, 195, 5, 16, 700, 0, 1, 1, 4, 64, 4, 64, "bf16", 65)
    _run_update_first(w, 7, meta16)


def test_update_first_order_vggt_layer():
    _run_update_first(si.WORKLOADS["vggt_layer"], 10, False)
