"""GPU checks at the full shapes of the benchmark's configurations, in the launch configurations bench.py
times: the bf16 output store on the one-layer workload, 24 frames of the 24-layer stack, 1000 frames of the
long stream (invariants), and the 4-stream x 24-layer high-resolution batch."""
import numpy as np
import pytest

import synth_inputs as si
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def test_vggt_layer_bf16_store_is_the_rounded_fp32_result_and_matches_the_oracle():
    """What bench.py times on one layer is the bf16 output store: on the vggt_layer shape it is bit for bit the
    nearest-even rounding of the fp32 output, and that fp32 output is within the tolerance of the oracle."""
    import torch
    import paper_2601_01204_amd as kvx
    from oracle import xstream_oracle as xo
    w = si.WORKLOADS["vggt_layer"]
    h32 = pu.make_handle(w, out_dtype=kvx.KV_F32)
    h16 = pu.make_handle(w, out_dtype=kvx.KV_BF16)
    cache = xo.OracleCache(pu.oracle_cfg(w))
    sigma = si.key_channel_scales(w)
    for t in range(11):                          # pruning starts at the 8th frame
        q, k, v = si.frame_qkv(w, t, sigma=sigma)
        ref = cache.step(q, k, v)
        tq, tk, tv = (pu.to_device(a, w) for a in (q, k, v))
        o32 = torch.empty(tq.shape, dtype=torch.float32, device=tq.device)
        o16 = torch.empty_like(tq)
        h32.step(tq, tk, tv, o32)
        h16.step(tq, tk, tv, o16)
        torch.cuda.synchronize()
        assert torch.equal(o32.to(torch.bfloat16), o16), f"frame {t}"
        pu.check_output(o32.cpu().numpy(), ref, f"vggt_layer frame {t}")
        # the bf16 values themselves: within half a bf16 unit of the oracle plus the fp32 path's own error
        got = o16.float().cpu().numpy().astype(np.float64)
        rms = float(np.sqrt((ref ** 2).mean()))
        assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -8 + 2e-2 * rms), f"frame {t}"
    pu.check_state(h16.export(), cache, "vggt_layer bf16-out handle")
    h32.close()
    h16.close()


def test_vggt_stack_24_frames_two_layers_against_the_oracle():
    """Budget 16384, all 24 layer caches per kv_step_batched call, 24 frames (pruning from the 16th): layers 3 and
    20 against their own oracles, every other layer twinned with one of them bit for bit."""
    import torch
    from oracle import xstream_oracle as xo
    w = si.WORKLOADS["vggt_stack"]
    layers = [3, 20]
    twin = {l: (3 if l % 2 else 20) for l in range(24)}
    h = pu.make_handle(w, n_layers=24)
    caches = {l: xo.OracleCache(pu.oracle_cfg(w)) for l in layers}
    sig = {l: si.key_channel_scales(w, 0, l) for l in layers}
    for t in range(24):
        dev, ref = {}, {}
        for l in layers:
            q, k, v = si.frame_qkv(w, t, 0, l, sig[l])
            ref[l] = caches[l].step(q, k, v)
            dev[l] = tuple(pu.to_device(a, w) for a in (q, k, v))
        outs = [torch.empty(dev[3][0].shape, dtype=torch.float32, device="cuda:0") for _ in range(24)]
        h.step_batched([(0, l, *dev[twin[l]], outs[l]) for l in range(24)])
        torch.cuda.synchronize()
        for l in layers:
            e = pu.check_output(outs[l].cpu().numpy(), ref[l], f"stack layer {l} frame {t}")
            if t >= 15 and t % 2 == 1:
                pu.check_state(h.export(0, l), caches[l], f"stack layer {l} frame {t}")
        for l in range(24):
            assert torch.equal(outs[l], outs[twin[l]]), f"layer {l} frame {t}"
        print(f"  stack frame {t}: len {caches[3].cache_len} err {e}", flush=True)
    h.close()


def _device_ring(w, caches, ring, seed):
    import torch
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(seed)
    n, H, d = w.tokens_per_frame, w.n_heads, w.head_dim
    out = []
    for _ in range(caches):
        sigma = torch.exp(torch.randn((H, d), generator=gen, device="cuda:0"))
        q = torch.randn((ring, n, H, d), generator=gen, device="cuda:0").to(torch.bfloat16)
        k = (torch.randn((ring, n, H, d), generator=gen, device="cuda:0") * sigma).to(torch.bfloat16)
        v = torch.randn((ring, n, H, d), generator=gen, device="cuda:0").to(torch.bfloat16)
        out.append((q, k, v))
    return out


@pytest.mark.parametrize("meta_format", [0, 1])
def test_vggt_long_1000_frames_24_layers_stay_flat(meta_format):
    """The long-stream configuration at its real shape (1041 tokens x 16 heads, budget 16384, 24 layers, 1000
    frames): cache length min(t n, L), allocated bytes constant, tokens dropped as counted, finite outputs."""
    import torch
    import paper_2601_01204_amd as kvx
    w = si.WORKLOADS["vggt_long"]
    n, L, NL = w.tokens_per_frame, w.budget_tokens, w.n_layers
    h = pu.make_handle(w, n_layers=NL, out_dtype=kvx.KV_BF16, meta_format=meta_format)
    ring = _device_ring(w, NL, 20, 7)
    outs = [torch.empty((n, w.n_heads, w.head_dim), dtype=torch.bfloat16, device="cuda:0") for _ in range(NL)]
    alloc0 = h.stats()["bytes_allocated"]
    for t in range(1000):
        r = t % 20
        h.step_batched([(0, l, ring[l][0][r], ring[l][1][r], ring[l][2][r], outs[l]) for l in range(NL)])
        if t + 1 in (1, 16, 100, 500, 1000):
            torch.cuda.synchronize()
            st = h.stats()
            assert st["cache_len_min"] == st["cache_len_max"] == min((t + 1) * n, L), t
            assert st["bytes_allocated"] == alloc0
            assert st["frames_seen_total"] == NL * (t + 1)
            assert st["tokens_dropped_total"] == NL * max(0, (t + 1) * n - L)
            assert st["zp_range_warnings"] == 0 and st["nonfinite_flag"] == 0
            assert all(bool(torch.isfinite(o.float()).all()) for o in outs), t
            print(f"  long stream frame {t + 1}: len {st['cache_len_max']} allocated {st['bytes_allocated']}", flush=True)
    ex = h.export(0, 11)
    assert ex["cache_len"] == L and len(np.unique(ex["ids"])) == L
    assert np.array_equal(ex["ids"][:n], np.arange(n)) and np.array_equal(ex["ids"][-n:], 999 * n + np.arange(n))
    assert np.all(np.diff(ex["ids"]) > 0)
    h.close()


def test_vggt_hires_four_streams_24_layers_in_one_call():
    """The high-resolution configuration's batch: 4 streams x 24 layers = 96 caches in one kv_step_batched (two
    launch sets of 48), 1374 tokens per frame, budget 24576, INT2 keys in groups of 32.  Cache (2, 13) is compared
    with the oracle over 20 frames (pruning from the 18th); all 96 caches get the same inputs and must agree bit
    for bit with it."""
    import torch
    from oracle import xstream_oracle as xo
    w = si.WORKLOADS["vggt_hires"]
    h = pu.make_handle(w, n_streams=4, n_layers=24)
    cache = xo.OracleCache(pu.oracle_cfg(w))
    sig = si.key_channel_scales(w, 2, 13)
    shape = (w.tokens_per_frame, w.n_heads, w.head_dim)
    outs = {(s, l): torch.empty(shape, dtype=torch.float32, device="cuda:0") for s in range(4) for l in range(24)}
    for t in range(20):
        q, k, v = si.frame_qkv(w, t, 2, 13, sig)
        ref = cache.step(q, k, v)
        dq, dk, dv = (pu.to_device(a, w) for a in (q, k, v))
        h.step_batched([(s, l, dq, dk, dv, outs[(s, l)]) for s in range(4) for l in range(24)])
        torch.cuda.synchronize()
        e = pu.check_output(outs[(2, 13)].cpu().numpy(), ref, f"hires frame {t}")
        for key, o in outs.items():
            assert torch.equal(o, outs[(2, 13)]), f"cache {key} frame {t}"
        if t >= 16:
            pu.check_state(h.export(2, 13), cache, f"hires frame {t}")
            a_ = h.export(2, 13)
            for key in ((0, 0), (3, 23), (1, 7)):
                b_ = h.export(*key)
                for name in ("ids", "k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero", "last_keep", "last_scores"):
                    if a_[name] is None:
                        assert b_[name] is None
                    else:
                        assert np.array_equal(a_[name].view(np.uint8), b_[name].view(np.uint8)), f"cache {key} frame {t}: {name}"
        print(f"  hires batch frame {t}: len {cache.cache_len} err {e}", flush=True)
    st = h.stats()
    assert st["n_caches"] == 96 and st["cache_len_min"] == st["cache_len_max"] == w.budget_tokens
    h.close()
