"""GPU parity at the edges of the configuration space: the largest budget the library
accepts, every head count class, frames smaller than one query block and budgets smaller
than one key group, explicit key-range split counts, more caches than one launch holds,
and a stream restarted with kv_reset.  Same bar as the other parity tests: integers and
fp32 bits exact, attention output within the tolerance (through the C ABI)."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import xstream_oracle as xo
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def test_maximum_budget():
    """budget_tokens = 32768, the cap: 32248 middle tokens, so the selection kernel holds its full
    32 keys per thread; the cache fills at the 64th frame and is pruned three times."""
    w = si.Workload("max_budget", 2, 64, 520, 5, 16, 32768, 68, 1, 1, 4, 64, 4, 64, "bf16", 21)
    quiet = lambda *a, **k: None
    pu.run_stream(w, 67, check_every=9, log=quiet)


@pytest.mark.parametrize("n_heads,n,budget", [(1, 77, 300), (5, 40, 170), (64, 37, 150)])
def test_head_counts(n_heads, n, budget):
    """One head (no head sum), an odd count, and the most the library takes (64)."""
    w = si.Workload(f"heads{n_heads}", n_heads, 64, n, 3, 8, budget, 7, 1, 1, 4, 32, 4, 64, "bf16", 22)
    pu.run_stream(w, 7)


def test_frames_smaller_than_a_query_block_and_budget_smaller_than_a_key_group():
    """3 tokens per frame (one special + one pooled pair), budget 20: a single ragged key group,
    a single partly filled query block, k = 14."""
    w = si.Workload("threes", 2, 64, 3, 1, 2, 20, 12, 1, 1, 8, 64, 8, 64, "f32", 23)
    pu.run_stream(w, 12)


@pytest.mark.parametrize("splits", [1, 3, 16])
def test_explicit_split_counts(splits):
    """The key range cut into 1, 3 and 16 pieces (more pieces than some steps have tiles)."""
    w = si.Workload("splits", 3, 64, 195, 5, 16, 700, 6, 1, 1, 4, 64, 4, 64, "bf16", 24)
    h = pu.make_handle(w)
    h.set_option("attention_splits", splits)
    pu.run_stream(w, 6, handle=h)
    h.close()


def test_more_caches_than_one_launch_holds():
    """52 caches stepped by one kv_step_batched call (a launch takes 48), each against its own oracle."""
    import torch
    n_streams = 52
    w = si.Workload("many", 2, 64, 40, 3, 8, 100, 4, 1, n_streams, 4, 64, 4, 64, "bf16", 25)
    h = pu.make_handle(w, n_streams=n_streams)
    caches = [xo.OracleCache(pu.oracle_cfg(w)) for _ in range(n_streams)]
    sigmas = [si.key_channel_scales(w, s, 0) for s in range(n_streams)]
    for t in range(4):
        items, refs, keep_alive = [], [], []
        for s in range(n_streams):
            q, k, v = si.frame_qkv(w, t, s, 0, sigmas[s])
            refs.append(caches[s].step(q, k, v))
            tq, tk, tv = (pu.to_device(a, w) for a in (q, k, v))
            out = torch.empty(tq.shape, dtype=torch.float32, device=tq.device)
            keep_alive.append((tq, tk, tv, out))
            items.append((s, 0, tq, tk, tv, out))
        h.step_batched(items)
        torch.cuda.synchronize()
        for s in range(n_streams):
            pu.check_output(keep_alive[s][3].cpu().numpy(), refs[s], f"stream {s} frame {t}")
            if s % 7 == 0 or s >= 47:
                pu.check_state(h.export(s, 0), caches[s], f"stream {s} frame {t}")
    h.close()


def test_reset_restarts_a_stream():
    """After kv_reset a cache behaves like a new one (frame numbering and pruning start over)."""
    w = si.Workload("again", 2, 64, 69, 5, 16, 200, 5, 1, 1, 4, 64, 4, 64, "bf16", 26)
    h = pu.make_handle(w)
    pu.run_stream(w, 5, handle=h)
    h.reset()
    assert h.stats()["cache_len_max"] == 0
    pu.run_stream(w, 5, handle=h)
    h.close()


@pytest.mark.parametrize("n,n_special,g", [(20, 20, 4), (37, 5, 64), (33, 0, 33)])
def test_pooling_extremes(n, n_special, g):
    """Every token special (no pooled group at all), one short group that holds all patch tokens,
    and one group of exactly all tokens."""
    w = si.Workload(f"pool{n}_{n_special}_{g}", 2, 64, n, n_special, g, 4 * n + 7, 8, 1, 1, 4, 32, 4, 32, "bf16", 27)
    pu.run_stream(w, 8)


def test_two_handles_interleaved():
    """Two handles of different shapes alive at once, stepped alternately on the same stream."""
    wa = si.Workload("ha", 2, 64, 69, 5, 16, 200, 6, 1, 1, 4, 64, 4, 64, "bf16", 28)
    wb = si.Workload("hb", 3, 64, 45, 3, 8, 150, 6, 1, 1, 8, 32, 2, 32, "f32", 29)
    import torch
    ha, hb = pu.make_handle(wa), pu.make_handle(wb)
    ca, cb = xo.OracleCache(pu.oracle_cfg(wa)), xo.OracleCache(pu.oracle_cfg(wb))
    sa, sb = si.key_channel_scales(wa), si.key_channel_scales(wb)
    for t in range(6):
        outs = []
        for w, h, c, sg in ((wa, ha, ca, sa), (wb, hb, cb, sb)):
            q, k, v = si.frame_qkv(w, t, sigma=sg)
            ref = c.step(q, k, v)
            tq, tk, tv = (pu.to_device(x, w) for x in (q, k, v))
            out = torch.empty(tq.shape, dtype=torch.float32, device=tq.device)
            h.step(tq, tk, tv, out)
            outs.append((w, h, c, out, ref, (tq, tk, tv)))
        torch.cuda.synchronize()
        for w, h, c, out, ref, _ in outs:
            pu.check_output(out.cpu().numpy(), ref, f"{w.name} frame {t}")
            pu.check_state(h.export(), c, f"{w.name} frame {t}")
    ha.close()
    hb.close()


def test_fp32_inputs_with_bf16_output():
    """in_dtype fp32, out_dtype bf16: the output is the nearest-even bf16 of the fp32-output run."""
    import torch
    w = si.Workload("mixed", 2, 64, 50, 5, 16, 160, 5, 1, 1, 4, 64, 4, 64, "f32", 30)
    h32 = pu.make_handle(w)
    h16 = pu.make_handle(w, out_dtype=0)
    sigma = si.key_channel_scales(w)
    for t in range(5):
        q, k, v = si.frame_qkv(w, t, sigma=sigma)
        tq, tk, tv = (pu.to_device(x, w) for x in (q, k, v))
        o32 = torch.empty(tq.shape, dtype=torch.float32, device=tq.device)
        o16 = torch.empty(tq.shape, dtype=torch.bfloat16, device=tq.device)
        h32.step(tq, tk, tv, o32)
        # out shares the element strides of q: a bf16 [n, H, d] tensor has the same strides in elements
        h16.step(tq, tk, tv, o16)
        torch.cuda.synchronize()
        assert torch.equal(o32.to(torch.bfloat16), o16), f"frame {t}"
    h32.close()
    h16.close()
