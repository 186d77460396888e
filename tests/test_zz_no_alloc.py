"""kv_step_static, the step entry point that allocates nothing (attention partials in the library's
static device array), against kv_step on a twin handle: two calls in a row, the second on a smaller
input, so that the second call finds the first one's contents in the shared array."""
import numpy as np
import pytest

import synth_inputs as si
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _pair_run(w, frames, splits):
    """Step a kv_step handle and a kv_step_static handle through the same frames; outputs within the
    attention tolerance of each other and of the oracle, cache state bit for bit."""
    import torch
    from oracle import xstream_oracle as xo
    ha, hb = pu.make_handle(w), pu.make_handle(w)
    for h in (ha, hb):
        h.set_option("attention_splits", splits)        # several key-range splits, so the partial buffers are used
    cache = xo.OracleCache(pu.oracle_cfg(w))
    sigma = si.key_channel_scales(w)
    for t in range(frames):
        q, k, v = si.frame_qkv(w, t, sigma=sigma)
        ref = cache.step(q, k, v)
        tq, tk, tv = (pu.to_device(a, w) for a in (q, k, v))
        oa = torch.empty(tq.shape, dtype=torch.float32, device=tq.device)
        ob = torch.full(tq.shape, float("nan"), dtype=torch.float32, device=tq.device)
        ha.step(tq, tk, tv, oa)
        hb.step_static(tq, tk, tv, ob)
        torch.cuda.synchronize()
        a, b = oa.cpu().numpy(), ob.cpu().numpy()
        pu.check_output(b, ref, f"{w.name} static frame {t}")
        rms = float(np.sqrt((ref ** 2).mean()))
        d = np.abs(a.astype(np.float64) - b) / rms
        assert d.max() <= pu.OUT_MAX_ABS and d.mean() <= pu.OUT_MEAN_ABS, f"{w.name} frame {t}: kv_step vs kv_step_static {d.max()}"
        assert np.array_equal(a, b), f"{w.name} frame {t}: same kernels and split count must give the same bits"
        ea, eb = ha.export(), hb.export()
        pu.check_state(eb, cache, f"{w.name} static frame {t}")
        for name in ("ids", "k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero"):
            assert np.array_equal(ea[name].view(np.uint8), eb[name].view(np.uint8)), f"{w.name} frame {t}: {name}"
    ha.close()
    hb.close()


def test_static_scratch_step_matches_kv_step_twice_in_a_row():
    big = si.Workload("static_big", 4, 64, 300, 5, 16, 1000, 6, 1, 1, 4, 64, 4, 64, "bf16", 41)
    small = si.Workload("static_small", 2, 64, 133, 5, 16, 500, 6, 1, 1, 4, 64, 4, 64, "bf16", 42)
    _pair_run(big, 6, 4)
    _pair_run(small, 6, 3)


def test_static_scratch_step_rejects_frames_beyond_the_array():
    import torch
    import paper_2601_01204_amd as kvx
    w = si.Workload("static_too_big", 64, 64, 1041, 5, 16, 2112, 1, 1, 1, 4, 64, 4, 64, "bf16", 43)
    h = pu.make_handle(w)
    x = torch.zeros((w.tokens_per_frame, w.n_heads, w.head_dim), dtype=torch.bfloat16, device="cuda:0")
    o = torch.zeros(x.shape, dtype=torch.float32, device="cuda:0")
    with pytest.raises(kvx.KvError) as e:
        h.step_static(x, x, x, o)
    assert e.value.code == -3 and "static scratch" in str(e.value)
    assert h.stats()["frames_seen_total"] == 0          # nothing was launched, the cache is untouched
    h.step(x, x, x, o)                                   # the allocating entry point still takes it
    torch.cuda.synchronize()
    h.close()
