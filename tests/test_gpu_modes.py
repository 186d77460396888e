"""GPU tests of the remaining entry points and modes: batched steps, the uncompressed bf16
baseline cache, strided inputs, determinism, long-run invariants, error paths."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import xstream_oracle as xo
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _small(**kw):
    base = dict(name="small", n_heads=2, head_dim=64, tokens_per_frame=133, n_special=5, pool_group=16,
                budget_tokens=500, frames=8, n_layers=1, n_streams=1, k_bits=4, k_group=64, v_bits=4, v_group=64,
                dtype="bf16", seed=31)
    base.update(kw)
    return si.Workload(**base)


def test_batched_steps_match_per_cache_oracles():
    """kv_step_batched over 2 streams x 3 layers: each cache evolves exactly like its own oracle."""
    import torch
    w = _small(n_layers=3, n_streams=2)
    h = pu.make_handle(w, n_streams=2, n_layers=3)
    caches = {(s, l): xo.OracleCache(pu.oracle_cfg(w)) for s in range(2) for l in range(3)}
    sig = {k: si.key_channel_scales(w, *k) for k in caches}
    for t in range(7):
        items, refs, outs = [], {}, {}
        for (s, l), cache in caches.items():
            q, k, v = si.frame_qkv(w, t, s, l, sig[(s, l)])
            refs[(s, l)] = cache.step(q, k, v)
            tq, tk, tv = (pu.to_device(a, w) for a in (q, k, v))
            out = torch.empty(tq.shape, dtype=torch.float32, device=tq.device)
            outs[(s, l)] = out
            items.append((s, l, tq, tk, tv, out))
        h.step_batched(items)
        torch.cuda.synchronize()
        for key, cache in caches.items():
            pu.check_output(outs[key].cpu().numpy(), refs[key], f"batched frame {t} cache {key}")
            pu.check_state(h.export(*key), cache, f"batched frame {t} cache {key}")
    st = h.stats()
    assert st["n_caches"] == 6 and st["frames_seen_total"] == 42
    assert st["cache_len_min"] == st["cache_len_max"] == 500
    h.close()


def test_batched_caches_at_different_lengths():
    """Caches of one batch may be at different frame counts (one prunes, the other does not)."""
    import torch
    w = _small(n_streams=2)
    h = pu.make_handle(w, n_streams=2)
    caches = [xo.OracleCache(pu.oracle_cfg(w)) for _ in range(2)]
    sig = [si.key_channel_scales(w, s, 0) for s in range(2)]
    frame = [0, 0]

    def feed(streams):
        items, chk = [], []
        for s in streams:
            q, k, v = si.frame_qkv(w, frame[s], s, 0, sig[s])
            ref = caches[s].step(q, k, v)
            tq, tk, tv = (pu.to_device(a, w) for a in (q, k, v))
            out = torch.empty(tq.shape, dtype=torch.float32, device=tq.device)
            items.append((s, 0, tq, tk, tv, out))
            chk.append((s, out, ref))
            frame[s] += 1
        h.step_batched(items)
        torch.cuda.synchronize()
        for s, out, ref in chk:
            pu.check_output(out.cpu().numpy(), ref, f"stream {s} frame {frame[s] - 1}")
            pu.check_state(h.export(s, 0), caches[s], f"stream {s} frame {frame[s] - 1}")

    for _ in range(3):
        feed([0])                 # stream 0 runs ahead: 3 frames, 399 tokens
    for _ in range(4):
        feed([0, 1])              # stream 0 prunes from its 4th frame on, stream 1 is still filling
    h.close()


def test_uncompressed_baseline_matches_full_attention():
    """KV_UNCOMPRESSED_BF16: a growing bf16 cache, no pruning, no quantisation = plain Eq. 1."""
    import torch
    import paper_2601_01204_amd as kvx
    w = _small()
    h = pu.make_handle(w, mode=kvx.KV_UNCOMPRESSED_BF16, max_frames=6)
    sigma = si.key_channel_scales(w)
    frames = [si.frame_qkv(w, t, sigma=sigma) for t in range(6)]
    for t, (q, k, v) in enumerate(frames):
        tq, tk, tv = (pu.to_device(a, w) for a in (q, k, v))
        out = torch.empty(tq.shape, dtype=torch.float32, device=tq.device)
        h.step(tq, tk, tv, out)
        torch.cuda.synchronize()
        ref = xo.reference_full_attention(frames, t, 1.0 / 8.0)
        pu.check_output(out.cpu().numpy(), ref, f"uncompressed frame {t}")
    st = h.stats()
    assert st["cache_len_max"] == 6 * w.tokens_per_frame
    tq, tk, tv = (pu.to_device(a, w) for a in frames[0])
    with pytest.raises(kvx.KvError) as e:          # the cache is full: max_frames reached
        h.step(tq, tk, tv, torch.empty(tq.shape, dtype=torch.float32, device=tq.device))
    assert e.value.code == -4
    h.close()


def test_strided_inputs():
    """q, k, v, out as slices of a fused [n, 3 + 1, H, d] buffer (non-trivial token stride)."""
    import torch
    w = _small(frames=5)
    h = pu.make_handle(w, out_dtype=0)       # bf16 out so that out shares the element strides and the buffer
    cache = xo.OracleCache(pu.oracle_cfg(w))
    sigma = si.key_channel_scales(w)
    n, H, d = w.tokens_per_frame, w.n_heads, w.head_dim
    for t in range(5):
        q, k, v = si.frame_qkv(w, t, sigma=sigma)
        ref = cache.step(q, k, v)
        fused = torch.zeros((n, 4, H, d), dtype=torch.bfloat16, device="cuda:0")
        for j, a in enumerate((q, k, v)):
            fused[:, j] = pu.to_device(a, w)
        h.step(fused[:, 0], fused[:, 1], fused[:, 2], fused[:, 3])
        torch.cuda.synchronize()
        got = fused[:, 3].float().cpu().numpy()
        rms = float(np.sqrt((ref ** 2).mean()))
        # bf16 store: tolerance plus half a bf16 ulp of the value itself
        assert np.all(np.abs(got - ref) <= pu.OUT_MAX_ABS * rms + np.abs(ref) * 2.0 ** -8)
        pu.check_state(h.export(), cache, f"strided frame {t}")
    h.close()


def test_two_runs_are_bit_identical():
    import torch
    w = _small(frames=7)
    results = []
    for _ in range(2):
        h = pu.make_handle(w)
        sigma = si.key_channel_scales(w)
        outs = []
        for t in range(7):
            tq, tk, tv = (pu.to_device(a, w) for a in si.frame_qkv(w, t, sigma=sigma))
            out = torch.empty(tq.shape, dtype=torch.float32, device=tq.device)
            h.step(tq, tk, tv, out)
            outs.append(out)
        torch.cuda.synchronize()
        ex = h.export()
        results.append(([o.cpu().numpy() for o in outs], ex))
        h.close()
    for a, b in zip(results[0][0], results[1][0]):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    for key in ("ids", "k_codes", "v_codes", "k_zero", "v_zero"):
        assert np.array_equal(results[0][1][key], results[1][1][key])


def test_long_stream_memory_and_length_stay_flat():
    """1000 frames: the cache length sits at the budget, the footprint never changes, outputs stay finite."""
    import torch
    w = _small(tokens_per_frame=69, budget_tokens=256, n_heads=2)
    h = pu.make_handle(w)
    sigma = si.key_channel_scales(w)
    ring = [tuple(pu.to_device(a, w) for a in si.frame_qkv(w, t, sigma=sigma)) for t in range(16)]
    out = torch.empty(ring[0][0].shape, dtype=torch.float32, device="cuda:0")
    base = None
    for t in range(1000):
        h.step(*ring[t % 16], out)
        if t in (0, 3, 99, 499, 999):
            st = h.stats()
            base = base or st["bytes_allocated"]
            assert st["bytes_allocated"] == base
            assert st["cache_len_max"] == min((t + 1) * 69, 256)
            assert bool(torch.isfinite(out).all())
    st = h.stats()
    assert st["frames_seen_total"] == 1000
    assert st["tokens_dropped_total"] == 1000 * 69 - 256
    ex = h.export()
    assert np.array_equal(ex["ids"][:69], np.arange(69))
    assert np.array_equal(ex["ids"][-69:], 999 * 69 + np.arange(69))
    assert np.all(np.diff(ex["ids"]) > 0)
    h.reset()
    assert h.stats()["cache_len_max"] == 0
    h.close()


def test_step_argument_errors_leave_the_cache_untouched():
    import torch
    import paper_2601_01204_amd as kvx
    w = _small()
    h = pu.make_handle(w)
    q, k, v = (pu.to_device(a, w) for a in si.frame_qkv(w, 0))
    out = torch.empty(q.shape, dtype=torch.float32, device="cuda:0")
    with pytest.raises(kvx.KvError) as e:
        h.step(q, k, v, out, stream=1)
    assert e.value.code == -3
    with pytest.raises(kvx.KvError) as e:
        h.step(q, k, v, out, layer=-1)
    assert e.value.code == -3
    with pytest.raises(kvx.KvError) as e:                     # the same cache twice in one batch
        h.step_batched([(0, 0, q, k, v, out), (0, 0, q, k, v, out)])
    assert e.value.code == -1
    lib = kvx.load_library()
    rc = lib.kv_step(h._h, 0, 0, q.data_ptr() + 2, k.data_ptr(), v.data_ptr(), q.stride(0), q.stride(1), out.data_ptr(), None)
    assert rc == -1 and b"aligned" in lib.kv_last_error(h._h)
    rc = lib.kv_step(h._h, 0, 0, q.data_ptr(), k.data_ptr(), v.data_ptr(), 8, 8, out.data_ptr(), None)
    assert rc == -1
    assert h.stats()["frames_seen_total"] == 0
    h.step(q, k, v, out)
    torch.cuda.synchronize()
    assert h.stats()["frames_seen_total"] == 1
    h.close()


def test_machine_probes_report_plausible_rates():
    """kv_probe_mfma_bf16 / kv_probe_copy: positive rates below the published peaks; bad arguments rejected."""
    import ctypes as C
    import paper_2601_01204_amd as kvx
    t = kvx.probe_mfma_bf16(2000, 2)
    assert 100.0 < t < 2600.0, t
    g = kvx.probe_copy(64 << 20, 2)
    assert 200.0 < g < 8500.0, g
    out = C.c_double(0.0)
    lib = kvx.load_library()
    assert lib.kv_probe_mfma_bf16(0, 1, None, C.byref(out)) == -1
    assert lib.kv_probe_copy(100, 1, None, C.byref(out)) == -1
    assert lib.kv_probe_copy(1 << 20, 1, None, None) == -1


def test_import_resumes_a_stream_bit_for_bit():
    """kv_export -> kv_import into a second handle: both continue the stream with identical outputs
    and cache states (the checkpoint holds everything a stream needs), and both still match the oracle."""
    import torch
    w = _small(frames=12)
    a = pu.make_handle(w)
    cache = xo.OracleCache(pu.oracle_cfg(w))
    sigma = si.key_channel_scales(w)
    frames = [si.frame_qkv(w, t, sigma=sigma) for t in range(12)]

    def feed(h, t):
        tq, tk, tv = (pu.to_device(x, w) for x in frames[t])
        out = torch.empty(tq.shape, dtype=torch.float32, device=tq.device)
        h.step(tq, tk, tv, out)
        torch.cuda.synchronize()
        return out.cpu().numpy()

    for t in range(8):                       # past pruning onset
        feed(a, t)
        cache.step(*frames[t])
    snap = a.export()
    b = pu.make_handle(w)
    b.import_state(snap)
    again = b.export()
    for name in ("ids", "k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero"):
        assert np.array_equal(snap[name].view(np.uint8), again[name].view(np.uint8)), name
    assert again["frames_seen"] == 8 and again["cache_len"] == snap["cache_len"]
    for t in range(8, 12):
        oa, ob = feed(a, t), feed(b, t)
        ref = cache.step(*frames[t])
        assert np.array_equal(oa.view(np.uint32), ob.view(np.uint32)), f"frame {t}: outputs differ after import"
        pu.check_output(ob, ref, f"imported frame {t}")
        pu.check_state(b.export(), cache, f"imported frame {t}")
    # inconsistent buffers are refused and leave the cache as it was
    bad = dict(snap)
    bad["frames_seen"] = 1
    with pytest.raises(kvx_mod().KvError) as e:
        b.import_state(bad)
    assert e.value.code == -1
    bad = dict(snap)
    bad["k_codes"] = snap["k_codes"].copy()
    bad["k_codes"][0, 0, 0] = 255
    with pytest.raises(kvx_mod().KvError):
        b.import_state(bad)
    pu.check_state(b.export(), cache, "after refused imports")
    a.close()
    b.close()


def kvx_mod():
    import paper_2601_01204_amd as kvx
    return kvx


def test_debug_checks_and_zero_point_warnings():
    """With "debug_checks" on, a NaN in k raises kv_stats' nonfinite_flag (clean inputs do not); a key channel far
    from zero in units of its range is counted in zp_range_warnings."""
    import torch
    w = _small(frames=4, dtype="f32")        # fp32 inputs: a range of 2^-9 at an offset of 2^12 needs 22 significant bits
    h = pu.make_handle(w)
    h.set_option("debug_checks", 1)
    sigma = si.key_channel_scales(w)
    q, k, v = si.frame_qkv(w, 0, sigma=sigma)
    tq, tk, tv = (pu.to_device(x, w) for x in (q, k, v))
    out = torch.empty(tq.shape, dtype=torch.float32, device=tq.device)
    h.step(tq, tk, tv, out)
    st = h.stats()
    assert st["nonfinite_flag"] == 0 and st["zp_range_warnings"] == 0
    k2 = k.copy()
    k2[:, 0, 3] = 4096.0 + 2.0 ** -9 * (np.arange(k.shape[0]) % 2)      # z = -4096 * 15 * 512, far beyond 2^20
    h.step(tq, pu.to_device(k2, w), tv, out)
    st = h.stats()
    assert st["nonfinite_flag"] == 0 and st["zp_range_warnings"] > 0
    k3 = k.copy()
    k3[5, 1, 7] = np.nan
    h.step(tq, pu.to_device(k3, w), tv, out)
    assert h.stats()["nonfinite_flag"] == 1
    h.close()


def test_timing_can_be_sampled():
    """kv_set_timing brackets every launch of the chosen classes, or those of every n-th step with "timing_every"."""
    import torch
    w = _small(frames=8)
    h = pu.make_handle(w)
    sigma = si.key_channel_scales(w)
    tq, tk, tv = (pu.to_device(x, w) for x in si.frame_qkv(w, 0, sigma=sigma))
    out = torch.empty(tq.shape, dtype=torch.float32, device=tq.device)
    h.set_timing(1 | (1 << 5))                 # attention and key rebuild
    for _ in range(8):
        h.step(tq, tk, tv, out)
    tm = h.read_timing()
    assert tm["attention"][1] == 8 and tm["rebuild_k"][1] == 8 and tm["score"][1] == 0
    assert tm["attention"][0] > 0.0
    h.set_option("timing_every", 4)
    for _ in range(8):
        h.step(tq, tk, tv, out)
    tm = h.read_timing()
    assert tm["attention"][1] == 2 and tm["rebuild_k"][1] == 2
    with pytest.raises(kvx_mod().KvError):
        h.set_option("timing_every", 0)
    h.close()
