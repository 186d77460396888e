"""Streams of different frame sizes in one handle (kv_set_stream_tokens): the token count of a frame follows the
video's aspect ratio (paper Sec. 4: maximum edge 518 pixels), so T_first, T_current, k and N_pooled of Sec. 3.2 are
those of the stream.  Each stream against its own oracle, same bars as everywhere."""
import dataclasses

import numpy as np
import pytest

import synth_inputs as si
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _run_two_streams(w_max, n_other, frames, meta16=False, slots=False):
    import torch
    from oracle import xstream_oracle as xo
    ws = [w_max, dataclasses.replace(w_max, tokens_per_frame=n_other, name=w_max.name + "_narrow")]
    h = pu.make_handle(w_max, n_streams=2, meta_format=1 if meta16 else 0, layout=1 if slots else 0)
    h.set_stream_tokens(1, n_other)
    caches = [xo.OracleCache(pu.oracle_cfg(w, meta16, slots)) for w in ws]
    sig = [si.key_channel_scales(ws[s], s, 0) for s in range(2)]
    for t in range(frames):
        for s in (0, 1):
            q, k, v = si.frame_qkv(ws[s], t, s, 0, sig[s])
            ref = caches[s].step(q, k, v)
            tq, tk, tv = (pu.to_device(a, ws[s]) for a in (q, k, v))
            out = torch.full(tq.shape, float("nan"), dtype=torch.float32, device=tq.device)
            h.step(tq, tk, tv, out, stream=s)
            torch.cuda.synchronize()
            e = pu.check_output(out.cpu().numpy(), ref, f"stream {s} frame {t}")
            pu.check_state(h.export(s, 0), caches[s], f"stream {s} frame {t}")
        print(f"  frame {t}: lens {caches[0].cache_len} {caches[1].cache_len} err {e}", flush=True)
    return h


@pytest.mark.parametrize("meta16,slots", [(False, False), (True, False), (False, True)])
def test_two_streams_of_different_frame_sizes(meta16, slots):
    w = si.Workload("wide", 3, 64, 195, 5, 16, 700, 0, 1, 2, 4, 64, 4, 64, "bf16", 81)
    h = _run_two_streams(w, 133, 9, meta16, slots)
    st = h.stats()
    assert st["cache_len_min"] == st["cache_len_max"] == 700
    h.close()


def test_frame_size_rules():
    import torch
    import paper_2601_01204_amd as kvx
    w = si.Workload("rules", 2, 64, 100, 5, 16, 400, 0, 2, 2, 4, 64, 4, 64, "bf16", 82)
    h = pu.make_handle(w, n_streams=2, n_layers=2)
    for bad in (0, 4, 101):
        with pytest.raises(kvx.KvError) as e:
            h.set_stream_tokens(1, bad)
        assert e.value.code == -3
    h.set_stream_tokens(1, 70)
    a = torch.zeros((100, 2, 64), dtype=torch.bfloat16, device="cuda:0")
    b = torch.zeros((70, 2, 64), dtype=torch.bfloat16, device="cuda:0")
    oa = torch.zeros(a.shape, dtype=torch.float32, device="cuda:0")
    ob = torch.zeros(b.shape, dtype=torch.float32, device="cuda:0")
    with pytest.raises(kvx.KvError) as e:           # one call carries frames of one size
        h.step_batched([(0, 0, a, a, a, oa), (1, 0, a, a, a, oa)])
    assert e.value.code == -1 and h.stats()["frames_seen_total"] == 0
    h.step_batched([(1, 0, b, b, b, ob), (1, 1, b, b, b, ob.clone())])       # both layers of the narrow stream
    h.step_batched([(0, 0, a, a, a, oa), (0, 1, a, a, a, oa.clone())])
    torch.cuda.synchronize()
    with pytest.raises(kvx.KvError) as e:           # the stream now holds frames
        h.set_stream_tokens(1, 80)
    assert e.value.code == -4
    h.reset(1, 0)
    h.reset(1, 1)
    h.set_stream_tokens(1, 80)
    ex = h.export(0, 1)
    assert ex["cache_len"] == 100
    h.close()


def test_vggt_scale_stream_of_782_tokens():
    """518 x 294 frames (37 x 21 patches + 5 = 782 tokens) in a handle sized for 1041: budget 8192, 14 frames
    (pruning from the 11th), against the oracle configured with n = 782."""
    import torch
    from oracle import xstream_oracle as xo
    w_max = si.WORKLOADS["vggt_layer"]
    w = dataclasses.replace(w_max, tokens_per_frame=782, name="vggt_782")
    h = pu.make_handle(w_max)
    h.set_stream_tokens(0, 782)
    pu.run_stream(w, 14, check_every=3, handle=h)
    assert h.stats()["tokens_dropped_total"] == 14 * 782 - 8192
    h.close()
