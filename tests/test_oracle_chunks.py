"""Pins for the oracle's multi-frame calls (frame-wise causal mask of Sec. 3.1 Eq. 1 inside a chunk, the chunk
appended as one block of current tokens) and for the update-first order (attend after prune).

Expected values come from a pure-Python masked softmax, from the equivalence with frame-by-frame stepping that
holds when nothing is pruned or quantised, from the printed Eq. 2-6 recomputed on the true keys by token id, and
from attention recomputed over exactly what the cache stores."""
import math

import numpy as np
import pytest

from oracle import xstream_oracle as xo


def _cfg(**kw):
    base = dict(n_heads=2, head_dim=16, tokens_per_frame=11, n_special=3, pool_group=4,
                budget_tokens=60, k_bits=8, k_group=8, v_bits=8, v_group=16)
    base.update(kw)
    return xo.OracleConfig(**base)


def _frames(cfg, count, seed=0):
    rng = np.random.default_rng(seed)
    sig = np.exp(rng.standard_normal((cfg.n_heads, cfg.head_dim))).astype(np.float32)
    shape = (cfg.tokens_per_frame, cfg.n_heads, cfg.head_dim)
    return [(rng.standard_normal(shape).astype(np.float32),
             (rng.standard_normal(shape).astype(np.float32) * sig).astype(np.float32),
             rng.standard_normal(shape).astype(np.float32)) for _ in range(count)]


def _chunk(frames):
    return tuple(np.concatenate([f[j] for f in frames], axis=0) for j in range(3))


def test_chunk_mask_against_pure_python_softmax():
    """Three frames of four tokens in one call on an empty cache: query i of frame a attends to the chunk's
    tokens 0 .. 4 (a + 1) - 1 and to nothing later, computed here with scalar loops."""
    cfg = _cfg(n_heads=1, head_dim=4, tokens_per_frame=4, n_special=1, pool_group=2, budget_tokens=100, quant=False, v_group=4)
    fr = _frames(cfg, 3, seed=2)
    q, k, v = _chunk(fr)
    out = xo.OracleCache(cfg).step(q, k, v)
    scale = 1.0 / math.sqrt(4)
    for i in range(12):
        vis = 4 * (i // 4 + 1)
        logits = [sum(float(q[i, 0, c]) * float(k[j, 0, c]) for c in range(4)) * scale for j in range(vis)]
        mx = max(logits)
        p = [math.exp(x - mx) for x in logits]
        tot = sum(p)
        for c in range(4):
            exp = sum(p[j] * float(v[j, 0, c]) for j in range(vis)) / tot
            assert abs(out[i, 0, c] - exp) < 1e-12
    # a later frame's key must not leak into an earlier frame's query: changing frame 2's keys leaves frames 0-1 unchanged
    k2 = k.copy()
    k2[8:] += 5.0
    out2 = xo.OracleCache(cfg).step(q, k2, v)
    assert np.array_equal(out2[:8], out[:8]) and not np.array_equal(out2[8:], out[8:])


@pytest.mark.parametrize("split", [(1, 1, 1, 1, 1, 1), (2, 1, 3), (6,), (3, 3)])
def test_chunks_equal_frame_by_frame_when_nothing_is_compressed(split):
    """No pruning, no quantisation: any grouping of the frames into calls gives the frame-by-frame outputs and state."""
    cfg = _cfg(budget_tokens=1000, quant=False)
    fr = _frames(cfg, 6, seed=3)
    ref_cache = xo.OracleCache(cfg)
    ref = np.concatenate([ref_cache.step(*f) for f in fr], axis=0)
    cache = xo.OracleCache(cfg)
    outs, t = [], 0
    for F in split:
        outs.append(cache.step(*_chunk(fr[t:t + F])))
        t += F
    got = np.concatenate(outs, axis=0)
    assert np.abs(got - ref).max() < 1e-12
    assert np.array_equal(cache.ids, ref_cache.ids) and np.array_equal(cache.K, ref_cache.K) and cache.frames == 6


def test_chunk_sees_the_cache_as_stored_and_its_own_frames_at_input_precision():
    """Quantised cache, no pruning: chunk frame a's output is Eq. 1 over [de-quantised cache before the call;
    chunk frames 0..a as given], recomputed here from the cache's stored values."""
    cfg = _cfg(budget_tokens=1000, k_bits=4, v_bits=4)
    fr = _frames(cfg, 5, seed=4)
    cache = xo.OracleCache(cfg)
    cache.step(*fr[0])
    cache.step(*fr[1])
    k_old, v_old = cache.stored_k().copy(), cache.stored_v().copy()
    q, k, v = _chunk(fr[2:5])
    out = cache.step(q, k, v)
    n = cfg.tokens_per_frame
    for a in range(3):
        ka = np.concatenate([k_old, k[:(a + 1) * n].transpose(1, 0, 2)], axis=1)
        va = np.concatenate([v_old, v[:(a + 1) * n].transpose(1, 0, 2)], axis=1)
        ref = xo.attention_fp64(q[a * n:(a + 1) * n], ka, va, 0.25)
        assert np.abs(out[a * n:(a + 1) * n] - ref).max() < 1e-12
    assert cache.frames == 5 and cache.cache_len == 5 * n
    assert cache.ids.tolist() == list(range(5 * n))


@pytest.mark.parametrize("F", [2, 3])
def test_chunk_pruning_keeps_first_frame_best_middle_and_the_whole_chunk(F):
    """Pruning only: after a chunk call the cache holds the first frame, the whole chunk and the k = L - n - F n
    best middle tokens, scored by Eq. 2-6 as printed with the pooled query rows of all F frames (recomputed here
    in fp64 on the true keys by token id)."""
    cfg = _cfg(quant=False, budget_tokens=58)
    fr = _frames(cfg, 3 + 4 * F, seed=30 + F)
    n, ns, g, L = cfg.tokens_per_frame, cfg.n_special, cfg.pool_group, cfg.budget_tokens
    all_k = np.concatenate([f[1] for f in fr], axis=0).astype(np.float64)
    cache = xo.OracleCache(cfg)
    for f in fr[:3]:
        cache.step(*f)
    t, pruned = 3, 0
    while t + F <= len(fr):
        ids_before = cache.ids.copy()
        q, k, v = _chunk(fr[t:t + F])
        cache.step(q, k, v)
        ids = np.concatenate([ids_before, t * n + np.arange(F * n)])
        T = len(ids)
        assert cache.cache_len == min(T, L)
        if T > L:
            pruned += 1
            q64 = q.astype(np.float64)
            rows = []
            for f in range(F):
                base = f * n
                rows += [q64[base + i] for i in range(ns)]
                a = ns
                while a < n:
                    rows.append(q64[base + a:base + min(a + g, n)].mean(axis=0))
                    a += g
            q_bar = np.stack(rows).mean(axis=1)
            mid_ids = ids[n:T - F * n]
            s = (q_bar @ all_k[mid_ids].mean(axis=1).T).mean(axis=0)
            kk = L - n - F * n
            order = np.argsort(-s, kind="stable")
            assert s[order[kk - 1]] - s[order[kk]] > 1e-4 * np.abs(s).max(), "near-tie in the test data"
            expect = np.concatenate([ids[:n], mid_ids[np.sort(order[:kk])], ids[T - F * n:]])
            assert np.array_equal(cache.ids, expect)
        t += F
    assert pruned >= 2


def test_single_frame_chunk_is_the_plain_step():
    cfg = _cfg(k_bits=4, v_bits=4, budget_tokens=40)
    fr = _frames(cfg, 7, seed=6)
    a, b = xo.OracleCache(cfg), xo.OracleCache(cfg)
    for f in fr:
        oa = a.step(*f)
        ob = b.step(*_chunk([f]))
        assert np.array_equal(oa, ob) and np.array_equal(a.Kc, b.Kc) and np.array_equal(a.ids, b.ids)


# ----------------------------------------------------------------------------- update first, then attend
@pytest.mark.parametrize("quant", [False, True])
def test_attend_after_prune_attends_over_exactly_the_stored_cache(quant):
    """The other order: the output of a step is Eq. 1 over the cache as it stands after the step (at most L_max
    keys, the current frame among them in stored form), recomputed here from the stored values; the cache itself
    evolves exactly as in the attend-first order, since the update never looks at the attention output."""
    cfg_a = _cfg(k_bits=4, v_bits=4, budget_tokens=40, quant=quant)
    cfg_b = _cfg(k_bits=4, v_bits=4, budget_tokens=40, quant=quant, attend_after_prune=True)
    fr = _frames(cfg_a, 8, seed=7)
    a, b = xo.OracleCache(cfg_a), xo.OracleCache(cfg_b)
    differ = 0
    for q, k, v in fr:
        oa = a.step(q, k, v)
        ob = b.step(q, k, v)
        assert np.array_equal(a.ids, b.ids)
        if quant:
            assert np.array_equal(a.Kc, b.Kc) and np.array_equal(a.Ks, b.Ks) and np.array_equal(a.Vc, b.Vc)
        assert b.cache_len <= 40
        ref = xo.attention_fp64(q, b.stored_k(), b.stored_v(), 0.25)
        assert np.abs(ob - ref).max() < 1e-12
        differ += int(np.abs(oa - ob).max() > 1e-6)
    assert differ >= 4          # once pruning (or quantisation of the current frame) bites, the two orders differ


def test_attend_after_prune_without_compression_is_full_attention():
    cfg = _cfg(budget_tokens=1000, quant=False, attend_after_prune=True)
    fr = _frames(cfg, 4, seed=8)
    cache = xo.OracleCache(cfg)
    for t, (q, k, v) in enumerate(fr):
        assert np.abs(cache.step(q, k, v) - xo.reference_full_attention(fr, t, 0.25)).max() < 1e-12
