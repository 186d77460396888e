"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the
same seeded inputs.  Kept indices, codes, scales and zero-points bit-exact; attention
output max abs <= 2e-2 and mean abs <= 2e-3 relative to unit-RMS outputs."""
import dataclasses

import numpy as np
import pytest

import synth_inputs as si
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def test_tiny_all_frames():
    """Configuration 'tiny': 8 frames, fp32 inputs, INT8/INT8, pruning from the 4th frame."""
    pu.run_stream(si.WORKLOADS["tiny"], 8)


@pytest.mark.parametrize("k_bits,k_group,v_bits,v_group,dtype", [
    (4, 64, 4, 64, "bf16"),
    (2, 32, 4, 64, "bf16"),
    (8, 64, 2, 32, "f32"),
    (4, 32, 8, 32, "bf16"),
    (2, 64, 2, 64, "f32"),
])
def test_small_mixed_formats(k_bits, k_group, v_bits, v_group, dtype):
    """Several tiles, ragged tails (n = 5 + 190 = 195, budget 700 not a multiple of 64)."""
    w = si.Workload("small", 3, 64, 195, 5, 16, 700, 7, 1, 1, k_bits, k_group, v_bits, v_group, dtype, 11)
    pu.run_stream(w, 7)


def test_budget_exactly_two_frames():
    """k = L_max - 2n = 0: only the first and the current frame survive."""
    w = si.Workload("two_frames", 2, 64, 70, 5, 16, 140, 5, 1, 1, 4, 64, 4, 64, "bf16", 12)
    pu.run_stream(w, 5)


def test_single_token_groups_and_no_specials():
    w = si.Workload("nospecial", 2, 64, 64, 0, 1, 200, 6, 1, 1, 4, 64, 4, 64, "f32", 13)
    pu.run_stream(w, 6)


def test_vggt_layer_first_frames():
    """The benchmark configuration (1041 tokens x 16 heads, budget 8192, INT4/INT4) across pruning onset."""
    w = si.WORKLOADS["vggt_layer"]
    pu.run_stream(w, 10, check_every=3)


def test_bf16_output_is_rounded_fp32_output():
    """The bf16 store is the fp32 result rounded to nearest-even: same kernels, same
    arithmetic, only the last conversion differs."""
    import torch
    import paper_2601_01204_amd as kvx
    w = si.Workload("small", 3, 64, 195, 5, 16, 700, 5, 1, 1, 4, 64, 4, 64, "bf16", 21)
    h32 = pu.make_handle(w, out_dtype=kvx.KV_F32)
    h16 = pu.make_handle(w, out_dtype=kvx.KV_BF16)
    sigma = si.key_channel_scales(w)
    for t in range(5):
        q, k, v = (pu.to_device(a, w) for a in si.frame_qkv(w, t, sigma=sigma))
        o32 = torch.empty(q.shape, dtype=torch.float32, device=q.device)
        o16 = torch.empty_like(q)
        h32.step(q, k, v, o32)
        h16.step(q, k, v, o16)
        torch.cuda.synchronize()
        assert torch.equal(o32.to(torch.bfloat16), o16), f"frame {t}"
    h32.close()
    h16.close()


def test_vggt_layer_all_frames():
    """All 32 frames of the benchmark configuration, free-running."""
    pu.run_stream(si.WORKLOADS["vggt_layer"], 32, check_every=8)


def test_vggt_hires_int2_keys_across_onset():
    """518x518 frames (1374 tokens), budget 24576, INT2 keys in groups of 32, INT4 values: 20 frames
    of one stream and layer (pruning starts at the 18th)."""
    w = si.WORKLOADS["vggt_hires"]
    pu.run_stream(w, 20, check_every=6)


def _run_custom_stream(w, frames_qkv):
    """Free-running parity on explicitly given frames."""
    import torch
    from oracle import xstream_oracle as xo
    h = pu.make_handle(w)
    cache = xo.OracleCache(pu.oracle_cfg(w))
    for t, (q, k, v) in enumerate(frames_qkv):
        ref = cache.step(q, k, v)
        tq, tk, tv = (pu.to_device(a, w) for a in (q, k, v))
        out = torch.empty(tq.shape, dtype=torch.float32, device=tq.device)
        h.step(tq, tk, tv, out)
        torch.cuda.synchronize()
        pu.check_output(out.float().cpu().numpy(), ref, f"{w.name} frame {t}")
        pu.check_state(h.export(), cache, f"{w.name} frame {t}")
    h.close()


def test_selection_with_tied_scores():
    """The same frame fed again and again: every middle token has duplicates with bit-identical
    scores, so the cut of the top-k falls inside runs of equal keys and the lower positions
    must win; the duplicated keys also give key groups whose codes repeat."""
    w = si.Workload("ties", 2, 64, 90, 5, 16, 400, 9, 1, 1, 4, 64, 4, 64, "bf16", 21)
    sigma = si.key_channel_scales(w)
    base = [si.frame_qkv(w, t, sigma=sigma) for t in range(2)]
    _run_custom_stream(w, [base[t % 2] for t in range(9)])


def test_zero_keys_give_signed_zero_scores_and_constant_groups():
    """Keys that are zero in whole frames and constant in others: scores of +0.0 / -0.0 (ordered
    -0 < +0 by the key image), groups with max == min (scale |min| or 1, code 0), and a cut
    through a run of equal scores."""
    w = si.Workload("zeros", 2, 64, 70, 5, 16, 300, 8, 1, 1, 4, 64, 4, 64, "f32", 22)
    sigma = si.key_channel_scales(w)
    frames = []
    for t in range(8):
        q, k, v = si.frame_qkv(w, t, sigma=sigma)
        if t in (1, 2):
            k = np.zeros_like(k)
        elif t == 3:
            k = np.full_like(k, -0.75)
        elif t == 4:
            k = np.zeros_like(k)
            k[:, :, ::2] = 0.5
        frames.append((q, k, v))
    _run_custom_stream(w, frames)
