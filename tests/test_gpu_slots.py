"""GPU parity for the slot-stable layout (KV_LAYOUT_SLOTS): tokens never move, freed slots take the new tokens,
key groups are re-quantised in place only when they received one.  Same bars as everywhere: kept indices, ids (in
slot order), scores, codes, scales and zero-points bit-exact, outputs within the attention tolerance."""
import dataclasses

import numpy as np
import pytest

import synth_inputs as si
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("meta16", [False, True])
@pytest.mark.parametrize("k_bits,k_group,v_bits,v_group", [(4, 64, 4, 64), (2, 32, 4, 32), (4, 32, 2, 64)])
def test_small_formats(meta16, k_bits, k_group, v_bits, v_group):
    w = si.Workload("slots", 3, 64, 195, 5, 16, 700, 9, 1, 1, k_bits, k_group, v_bits, v_group, "bf16", 71)
    pu.run_stream(w, 9, meta16=meta16, slots=True)


def test_fp32_inputs_eight_bit_codes_and_short_frames():
    w = si.Workload("slots32", 2, 64, 133, 5, 16, 500, 8, 1, 1, 8, 64, 8, 64, "f32", 72)
    pu.run_stream(w, 8, slots=True)
    w = si.Workload("slots_short", 5, 64, 3, 1, 2, 40, 30, 1, 1, 4, 64, 4, 64, "bf16", 73)
    pu.run_stream(w, 30, slots=True)
    w = si.Workload("slots_two", 2, 64, 70, 5, 16, 140, 5, 1, 1, 4, 64, 4, 64, "bf16", 74)      # k = 0
    pu.run_stream(w, 5, slots=True)


@pytest.mark.parametrize("meta16", [False, True])
def test_vggt_layer_across_onset(meta16):
    pu.run_stream(si.WORKLOADS["vggt_layer"], 12, check_every=3, meta16=meta16, slots=True)


def test_vggt_stack_batched_across_onset_and_footprint():
    """Budget 16384, 24 layer caches per kv_step_batched call, 19 frames; layer 9 against the oracle, the others
    twinned with it.  One buffer per cache: allocated bytes per cache stay within 1.15 x the live bytes plus the
    attention partials."""
    import torch
    from oracle import xstream_oracle as xo
    w = si.WORKLOADS["vggt_stack"]
    h = pu.make_handle(w, n_layers=24, layout=1)
    cache = xo.OracleCache(pu.oracle_cfg(w, False, True))
    sig = si.key_channel_scales(w, 0, 9)
    for t in range(19):
        q, k, v = si.frame_qkv(w, t, 0, 9, sig)
        ref = cache.step(q, k, v)
        dq, dk, dv = (pu.to_device(a, w) for a in (q, k, v))
        outs = [torch.empty(dq.shape, dtype=torch.float32, device=dq.device) for _ in range(24)]
        h.step_batched([(0, l, dq, dk, dv, outs[l]) for l in range(24)])
        torch.cuda.synchronize()
        e = pu.check_output(outs[9].cpu().numpy(), ref, f"slots stack frame {t}")
        for l in range(24):
            assert torch.equal(outs[l], outs[9]), f"layer {l} frame {t}"
        if t >= 14:
            pu.check_state(h.export(0, 9), cache, f"slots stack frame {t}")
            a_, b_ = h.export(0, 22), h.export(0, 9)
            for name in ("ids", "k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero"):
                assert np.array_equal(a_[name].view(np.uint8), b_[name].view(np.uint8)), f"layer 22 frame {t}: {name}"
        print(f"  slots stack frame {t}: len {cache.cache_len} err {e}", flush=True)
    st = h.stats()
    cache_bytes = st["bytes_k_codes"] + st["bytes_k_meta"] + st["bytes_v_codes"] + st["bytes_v_meta"] + st["bytes_ids"]
    assert cache_bytes <= 1.01 * 24 * st["bytes_live_per_cache"]
    h.close()


def test_chunks_and_update_first_on_slots():
    import torch
    import paper_2601_01204_amd as kvx
    from oracle import xstream_oracle as xo
    w = si.Workload("slots_chunks", 3, 64, 70, 5, 16, 500, 0, 1, 1, 4, 64, 4, 64, "bf16", 75)
    h = pu.make_handle(w, layout=1, max_frames_per_step=3)
    cache = xo.OracleCache(pu.oracle_cfg(w, False, True))
    sigma = si.key_channel_scales(w)
    t = 0
    for F in (2, 3, 1, 3, 3, 2, 3):
        fr = [si.frame_qkv(w, t + f, sigma=sigma) for f in range(F)]
        q, k, v = (np.concatenate([f[j] for f in fr], axis=0) for j in range(3))
        ref = cache.step(q, k, v)
        tq, tk, tv = (pu.to_device(a, w) for a in (q, k, v))
        out = torch.empty(tq.shape, dtype=torch.float32, device=tq.device)
        h.step_frames(F, tq, tk, tv, out)
        torch.cuda.synchronize()
        pu.check_output(out.cpu().numpy(), ref, f"slots chunk at frame {t}")
        pu.check_state(h.export(), cache, f"slots chunk at frame {t}")
        t += F
    h.close()
    w = si.Workload("slots_upd", 3, 64, 195, 5, 16, 700, 0, 1, 1, 4, 64, 4, 64, "bf16", 76)
    h = pu.make_handle(w, layout=1, order=kvx.KV_PRUNE_THEN_ATTEND)
    cache = xo.OracleCache(dataclasses.replace(pu.oracle_cfg(w, False, True), attend_after_prune=True))
    sigma = si.key_channel_scales(w)
    for t in range(7):
        q, k, v = si.frame_qkv(w, t, sigma=sigma)
        ref = cache.step(q, k, v)
        tq, tk, tv = (pu.to_device(a, w) for a in (q, k, v))
        out = torch.empty(tq.shape, dtype=torch.float32, device=tq.device)
        h.step(tq, tk, tv, out)
        torch.cuda.synchronize()
        pu.check_output(out.cpu().numpy(), ref, f"slots update-first frame {t}")
        pu.check_state(h.export(), cache, f"slots update-first frame {t}")
    h.close()


def test_import_and_long_run_on_slots():
    """Resume from an export bit for bit, then 300 frames: length and allocation flat, every token id unique,
    the first frame still in slots 0..n-1."""
    import torch
    w = si.Workload("slots_long", 2, 64, 69, 5, 16, 256, 0, 1, 1, 4, 64, 4, 64, "bf16", 77)
    ha, hb = pu.make_handle(w, layout=1), pu.make_handle(w, layout=1)
    sigma = si.key_channel_scales(w)
    frames = [tuple(pu.to_device(a, w) for a in si.frame_qkv(w, t, sigma=sigma)) for t in range(16)]
    oa = torch.empty(frames[0][0].shape, dtype=torch.float32, device="cuda:0")
    ob = torch.empty_like(oa)
    for t in range(6):
        ha.step(*frames[t], oa)
    torch.cuda.synchronize()
    hb.import_state(ha.export())
    alloc = ha.stats()["bytes_allocated"]
    for t in range(6, 300):
        ha.step(*frames[t % 16], oa)
        hb.step(*frames[t % 16], ob)
        if t < 12 or t == 299:
            torch.cuda.synchronize()
            assert torch.equal(oa, ob), f"frame {t}"
            ea, eb = ha.export(), hb.export()
            for name in ("ids", "k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero"):
                assert np.array_equal(ea[name].view(np.uint8), eb[name].view(np.uint8)), f"frame {t}: {name}"
    ex, st = ha.export(), ha.stats()
    assert st["cache_len_max"] == 256 and st["bytes_allocated"] == alloc
    assert len(np.unique(ex["ids"])) == 256 and np.array_equal(ex["ids"][:69], np.arange(69))
    assert set(range(299 * 69, 300 * 69)) <= set(ex["ids"].tolist())
    ha.close()
    hb.close()
