"""The stream contract of the boundary: a step is enqueued on the stream the caller names and never synchronises;
all calls on one handle must be ordered with each other (the handle's scratch and partial-result buffers are shared
by its caches).  Two caches of one handle stepped on two different non-default streams, with the order between
consecutive calls made explicit by events exactly as the contract asks, must evolve like their oracles; and a step
whose inputs are produced on its stream just before the call must see them."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import xstream_oracle as xo
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _w():
    return si.Workload(name="streams", n_heads=4, head_dim=64, tokens_per_frame=133, n_special=5, pool_group=16,
                       budget_tokens=500, frames=7, n_layers=2, n_streams=1, k_bits=4, k_group=64, v_bits=4, v_group=64,
                       dtype="bf16", seed=91)


@pytest.mark.parametrize("meta16,slots", [(False, False), (True, False), (True, True)])
def test_two_caches_on_two_streams_ordered_by_events(meta16, slots):
    import torch
    w = _w()
    h = pu.make_handle(w, n_layers=2, meta_format=1 if meta16 else 0, layout=1 if slots else 0)
    caches = [xo.OracleCache(pu.oracle_cfg(w, meta16, slots)) for _ in range(2)]
    sig = [si.key_channel_scales(w, 0, l) for l in range(2)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    last = None                                   # event after the previous call on the handle
    keep_alive, results = [], []
    for t in range(w.frames):
        for l in range(2):
            q, k, v = si.frame_qkv(w, t, 0, l, sig[l])
            ref = caches[l].step(q, k, v)
            s = streams[l]
            with torch.cuda.stream(s):
                # the inputs are uploaded and converted on the step's own stream, right before the call
                tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0").to(torch.bfloat16) for a in (q, k, v))
                out = torch.empty(tq.shape, dtype=torch.float32, device="cuda:0")
                if last is not None:
                    s.wait_event(last)            # the contract: calls on one handle are ordered with each other
                h.step(tq, tk, tv, out, stream=0, layer=l, hip_stream=s.cuda_stream)
                last = torch.cuda.Event()
                last.record(s)
            keep_alive.append((tq, tk, tv))        # nothing is freed or waited for until every call is enqueued
            results.append((t, l, out, ref))
    torch.cuda.synchronize()
    for t, l, out, ref in results:
        pu.check_output(out.cpu().numpy(), ref, f"frame {t} layer {l}")
    for l in range(2):
        pu.check_state(h.export(0, l), caches[l], f"final state of layer {l}")
    h.close()
