"""GPU parity with the 16-bit quantiser metadata format (KV_META_F16): the HIP path through the C ABI
against the oracle's meta16 variant.  Kept indices, scores, codes, scales (bits) and zero-points
bit-exact; attention output max abs <= 2e-2 and mean abs <= 2e-3 relative to unit-RMS outputs."""
import numpy as np
import pytest

import synth_inputs as si
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("k_bits,k_group,v_bits,v_group", [
    (4, 64, 4, 64),
    (2, 32, 4, 64),
    (4, 32, 8, 32),
    (2, 64, 2, 64),
    (4, 64, 2, 32),
])
def test_small_formats(k_bits, k_group, v_bits, v_group):
    """Several tiles, ragged tails (n = 5 + 190 = 195, budget 700 not a multiple of 64), pruning from the 4th frame."""
    w = si.Workload("small16", 3, 64, 195, 5, 16, 700, 7, 1, 1, k_bits, k_group, v_bits, v_group, "bf16", 51)
    pu.run_stream(w, 7, meta16=True)


def test_budget_exactly_two_frames_and_short_frames():
    w = si.Workload("two_frames16", 2, 64, 70, 5, 16, 140, 5, 1, 1, 4, 64, 4, 64, "bf16", 52)
    pu.run_stream(w, 5, meta16=True)
    w = si.Workload("short16", 5, 64, 3, 1, 2, 40, 20, 1, 1, 4, 64, 4, 64, "bf16", 53)
    pu.run_stream(w, 20, meta16=True)


def test_vggt_layer_across_onset():
    """1041 tokens x 16 heads, budget 8192, INT4/INT4, 12 frames (pruning starts at the 8th)."""
    pu.run_stream(si.WORKLOADS["vggt_layer"], 12, check_every=3, meta16=True)


def test_vggt_hires_int2_keys_across_onset():
    """1374 tokens per frame, budget 24576, INT2 keys in groups of 32: 20 frames of one cache."""
    pu.run_stream(si.WORKLOADS["vggt_hires"], 20, check_every=6, meta16=True)


def test_vggt_stack_batched_across_onset():
    """Budget 16384, all 24 layer caches per kv_step_batched call (the launch the benchmark times), 18 frames; layer 5
    runs its own inputs against the oracle, every other layer is fed the same inputs and must match it bit for bit."""
    import torch
    from oracle import xstream_oracle as xo
    w = si.WORKLOADS["vggt_stack"]
    h = pu.make_handle(w, n_layers=24, meta_format=1)
    cache = xo.OracleCache(pu.oracle_cfg(w, True))
    sig = si.key_channel_scales(w, 0, 5)
    for t in range(18):
        q, k, v = si.frame_qkv(w, t, 0, 5, sig)
        ref = cache.step(q, k, v)
        dq, dk, dv = (pu.to_device(a, w) for a in (q, k, v))
        outs = [torch.empty(dq.shape, dtype=torch.float32, device=dq.device) for _ in range(24)]
        h.step_batched([(0, l, dq, dk, dv, outs[l]) for l in range(24)])
        torch.cuda.synchronize()
        e = pu.check_output(outs[5].cpu().numpy(), ref, f"stack16 frame {t}")
        for l in range(24):
            assert torch.equal(outs[l], outs[5]), f"layer {l} frame {t}"
        if t >= 14:
            pu.check_state(h.export(0, 5), cache, f"stack16 frame {t}")
            a_, b_ = h.export(0, 17), h.export(0, 5)
            for name in ("ids", "k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero"):
                assert np.array_equal(a_[name].view(np.uint8), b_[name].view(np.uint8)), f"layer 17 frame {t}: {name}"
        print(f"  stack16 frame {t}: len {cache.cache_len} err {e}", flush=True)
    st = h.stats()
    # 4.5 bits per element: codes + 4 bytes per group
    H, L, d = w.n_heads, w.budget_tokens, w.head_dim
    assert st["bytes_live_per_cache"] == 2 * (H * L * d // 2) + H * (L // 64) * d * 4 + H * L * 4 + L * 4
    h.close()


def test_import_resumes_bit_for_bit():
    import torch
    w = si.Workload("imp16", 2, 64, 133, 5, 16, 500, 9, 1, 1, 4, 64, 4, 64, "bf16", 54)
    ha = pu.make_handle(w, meta_format=1)
    hb = pu.make_handle(w, meta_format=1)
    sigma = si.key_channel_scales(w)
    frames = [tuple(pu.to_device(a, w) for a in si.frame_qkv(w, t, sigma=sigma)) for t in range(9)]
    oa = torch.empty(frames[0][0].shape, dtype=torch.float32, device="cuda:0")
    ob = torch.empty_like(oa)
    for t in range(6):
        ha.step(*frames[t], oa)
    torch.cuda.synchronize()
    hb.import_state(ha.export())
    for t in range(6, 9):
        ha.step(*frames[t], oa)
        hb.step(*frames[t], ob)
        torch.cuda.synchronize()
        assert torch.equal(oa, ob), f"frame {t}"
        ea, eb = ha.export(), hb.export()
        for name in ("ids", "k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero", "last_keep", "last_scores"):
            assert np.array_equal(ea[name].view(np.uint8), eb[name].view(np.uint8)), f"frame {t}: {name}"
    ha.close()
    hb.close()


def test_scales_below_the_half_range_are_kept_inside_and_counted():
    """Keys 4096 times smaller than usual: the logit-domain scale of most groups falls below the smallest normal
    half and is held at 2^-14 (oracle and kernel alike), the groups are counted in zp_range_warnings; outputs and
    state still match the oracle.  (The upper end, 2048, lies beyond keys the half-precision products can hold.)"""
    import torch
    from oracle import xstream_oracle as xo
    w = si.Workload("sat16", 2, 64, 70, 5, 16, 300, 5, 1, 1, 4, 64, 4, 64, "bf16", 55)
    h = pu.make_handle(w, meta_format=1)
    cache = xo.OracleCache(pu.oracle_cfg(w, True))
    sigma = si.key_channel_scales(w)
    for t in range(5):
        q, k, v = si.frame_qkv(w, t, sigma=sigma)
        k = si.round_to_bf16(k * np.float32(2.0 ** -12))
        ref = cache.step(q, k, v)
        tq, tk, tv = (pu.to_device(a, w) for a in (q, k, v))
        out = torch.empty(tq.shape, dtype=torch.float32, device=tq.device)
        h.step(tq, tk, tv, out)
        torch.cuda.synchronize()
        pu.check_output(out.cpu().numpy(), ref, f"sat16 frame {t}")
        pu.check_state(h.export(), cache, f"sat16 frame {t}")
    assert np.any(cache.Ks == np.float32(np.float32(2.0 ** -14) * np.float32(np.float32(1.0) / xo.logit_scale_log2(0.125))))
    assert h.stats()["zp_range_warnings"] > 0
    h.close()
