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
