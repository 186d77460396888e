"""The three stream schedules of a step (option "overlap_update": 0 everything in order on the caller's stream,
1 the library's choice, 2 the update chain on the library's second stream at any launch size) only reorder
independent kernels: every one of them must leave bit-identical caches and outputs, on one cache per call (a launch
that cannot fill the chip) and on a batch whose attention launch has more workgroup columns than the chip has compute
units, in both layouts.  Schedule 1 of the same streams is compared with the oracle here as well."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import xstream_oracle as xo
from tests import parity_util as pu

pytestmark = pytest.mark.gpu

STATE_KEYS = ("ids", "k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero", "last_keep", "last_scores")


def _w(**kw):
    base = dict(name="sched", n_heads=16, head_dim=64, tokens_per_frame=69, n_special=5, pool_group=16,
                budget_tokens=256, frames=8, n_layers=1, n_streams=1, k_bits=4, k_group=64, v_bits=4, v_group=64,
                dtype="bf16", seed=77)
    base.update(kw)
    return si.Workload(**base)


def _same_export(a, b, what):
    assert a["cache_len"] == b["cache_len"], what
    for k in STATE_KEYS:
        if a[k] is None or b[k] is None:
            assert a[k] is None and b[k] is None, f"{what}: {k}"
            continue
        x, y = np.asarray(a[k]), np.asarray(b[k])
        if x.dtype.kind == "f":
            x, y = x.view(np.uint32), y.view(np.uint32)
        assert np.array_equal(x, y), f"{what}: {k} differs between schedules"


@pytest.mark.parametrize("slots", [False, True])
@pytest.mark.parametrize("n_layers", [1, 24])
def test_every_schedule_gives_the_same_bits(n_layers, slots):
    import torch
    w = _w(n_layers=n_layers)
    # 24 caches x 16 heads x 1 query tile = 384 workgroup columns: more than the 256 compute units
    handles = []
    for mode in (0, 1, 2):
        h = pu.make_handle(w, n_layers=n_layers, meta_format=1, layout=1 if slots else 0)
        h.set_option("overlap_update", mode)
        handles.append(h)
    checked = (0, n_layers - 1) if n_layers > 1 else (0,)
    caches = {l: xo.OracleCache(pu.oracle_cfg(w, True, slots)) for l in checked}
    sig = [si.key_channel_scales(w, 0, l) for l in range(n_layers)]
    for t in range(w.frames):                     # pruning starts at the fourth frame
        frames = [si.frame_qkv(w, t, 0, l, sig[l]) for l in range(n_layers)]
        dev = [tuple(pu.to_device(a, w) for a in f) for f in frames]
        refs = {l: caches[l].step(*frames[l]) for l in checked}
        outs = []
        for h in handles:
            o = [torch.empty(dev[l][0].shape, dtype=torch.float32, device="cuda:0") for l in range(n_layers)]
            h.step_batched([(0, l, dev[l][0], dev[l][1], dev[l][2], o[l]) for l in range(n_layers)])
            outs.append(o)
        torch.cuda.synchronize()
        for l in range(n_layers):
            a = outs[0][l].cpu().numpy().view(np.uint32)
            for m in (1, 2):
                assert np.array_equal(a, outs[m][l].cpu().numpy().view(np.uint32)), f"frame {t} layer {l}: outputs of schedules 0 and {m} differ"
        for l in checked:
            pu.check_output(outs[1][l].cpu().numpy(), refs[l], f"frame {t} layer {l}")
            ex = [h.export(0, l) for h in handles]
            pu.check_state(ex[1], caches[l], f"frame {t} layer {l}")
            _same_export(ex[0], ex[1], f"frame {t} layer {l} schedules 0/1")
            _same_export(ex[0], ex[2], f"frame {t} layer {l} schedules 0/2")
    for h in handles:
        h.close()
