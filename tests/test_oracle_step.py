"""Whole-step pins for the oracle: the streaming step against un-pruned,
un-quantised attention, and the invariants the paper states (bounded cache,
first and current frames kept, k = max(0, L_max - T_first - T_current))."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import xstream_oracle as xo


def _small_cfg(**kw):
    base = dict(n_heads=2, head_dim=16, tokens_per_frame=11, n_special=3, pool_group=4,
                budget_tokens=40, k_bits=8, k_group=8, v_bits=8, v_group=16)
    base.update(kw)
    return xo.OracleConfig(**base)


def _frames(cfg, count, seed=0, outliers=True):
    rng = np.random.default_rng(seed)
    sig = np.exp(rng.standard_normal((cfg.n_heads, cfg.head_dim))).astype(np.float32) if outliers else 1.0
    shape = (cfg.tokens_per_frame, cfg.n_heads, cfg.head_dim)
    return [(rng.standard_normal(shape).astype(np.float32),
             (rng.standard_normal(shape).astype(np.float32) * sig).astype(np.float32),
             rng.standard_normal(shape).astype(np.float32)) for _ in range(count)]


def test_no_compression_reproduces_full_attention():
    """quant off and a budget >= all tokens: every step is plain Eq. 1 over all frames."""
    cfg = _small_cfg(budget_tokens=1000, quant=False)
    fr = _frames(cfg, 5)
    cache = xo.OracleCache(cfg)
    for t, (q, k, v) in enumerate(fr):
        out = cache.step(q, k, v)
        ref = xo.reference_full_attention(fr, t, 1.0 / np.sqrt(cfg.head_dim))
        assert np.abs(out - ref).max() < 1e-12
        assert cache.cache_len == (t + 1) * cfg.tokens_per_frame


def test_pruning_only_equals_attention_over_kept_ids():
    """quant off, finite budget: each step's output is Eq. 1 over exactly the tokens
    whose ids the cache held before the step, plus the frame's own."""
    cfg = _small_cfg(quant=False)
    fr = _frames(cfg, 8, seed=1)
    n = cfg.tokens_per_frame
    all_k = np.concatenate([f[1] for f in fr], axis=0)     # [frames*n, H, d] indexed by token id
    all_v = np.concatenate([f[2] for f in fr], axis=0)
    cache = xo.OracleCache(cfg)
    for t, (q, k, v) in enumerate(fr):
        ids_before = cache.ids.copy()
        out = cache.step(q, k, v)
        ids = np.concatenate([ids_before, t * n + np.arange(n)])
        ka = all_k[ids].transpose(1, 0, 2)
        va = all_v[ids].transpose(1, 0, 2)
        ref = xo.attention_fp64(q, ka, va, 1.0 / np.sqrt(cfg.head_dim))
        assert np.abs(out - ref).max() < 1e-12


@pytest.mark.parametrize("budget", [22, 23, 40, 57, 200])
def test_cache_invariants(budget):
    cfg = _small_cfg(budget_tokens=budget, k_bits=4, v_bits=4)
    n = cfg.tokens_per_frame
    fr = _frames(cfg, 9, seed=budget)
    cache = xo.OracleCache(cfg)
    for t, (q, k, v) in enumerate(fr):
        T_before = cache.cache_len
        cache.step(q, k, v)
        T = T_before + n
        assert cache.cache_len == min(T, budget)
        assert cache.cache_len <= budget
        ids = cache.ids
        assert np.all(np.diff(ids) > 0)
        assert np.array_equal(ids[:n], np.arange(n))                          # first frame kept
        assert np.array_equal(ids[-n:], t * n + np.arange(n))                 # current frame kept
        if T > budget:
            keep = cache.last_keep
            assert len(keep) == budget
            k_top = budget - 2 * n
            assert len(keep) - 2 * n == k_top
            # the kept middle tokens are the k best: no dropped score beats a kept one
            s = cache.last_scores
            kept_mid = keep[n:len(keep) - n] - n
            dropped = np.setdiff1d(np.arange(len(s)), kept_mid)
            if len(kept_mid) and len(dropped):
                assert s[kept_mid].min() >= s[dropped].max()
        else:
            assert cache.last_keep is None
        # state sizes depend only on the cache length
        Tn = cache.cache_len
        G = cfg.k_group
        assert cache.Kc.shape == (cfg.n_heads, Tn, cfg.head_dim)
        assert cache.Ks.shape == (cfg.n_heads, -(-Tn // G), cfg.head_dim)
        assert cache.Vs.shape == (cfg.n_heads, Tn, cfg.head_dim // cfg.v_group)
        assert cache.Kc.max() <= 15 and cache.Vc.max() <= 15


def test_budget_below_two_frames_keeps_first_and_current_only():
    cfg = _small_cfg(budget_tokens=15, quant=False)
    n = cfg.tokens_per_frame
    fr = _frames(cfg, 4, seed=3)
    cache = xo.OracleCache(cfg)
    for t, f in enumerate(fr):
        cache.step(*f)
        if t >= 1:
            assert cache.ids.tolist() == list(range(n)) + list(range(t * n, (t + 1) * n))


def test_eight_bit_cache_close_to_full_precision():
    cfg = _small_cfg(budget_tokens=1000)
    fr = _frames(cfg, 4, seed=4)
    cache = xo.OracleCache(cfg)
    for t, f in enumerate(fr):
        out = cache.step(*f)
        ref = xo.reference_full_attention(fr, t, 1.0 / np.sqrt(cfg.head_dim))
        assert np.abs(out - ref).max() < 0.05
    # four-bit is visibly worse than eight-bit but still bounded
    cache4 = xo.OracleCache(_small_cfg(budget_tokens=1000, k_bits=4, v_bits=4))
    worst8, worst4 = 0.0, 0.0
    cache8 = xo.OracleCache(cfg)
    for t, f in enumerate(fr):
        ref = xo.reference_full_attention(fr, t, 1.0 / np.sqrt(cfg.head_dim))
        worst8 = max(worst8, np.abs(cache8.step(*f) - ref).max())
        worst4 = max(worst4, np.abs(cache4.step(*f) - ref).max())
    assert worst8 < worst4 < 1.0


def test_stored_values_within_half_a_step():
    """Right after a token's group is (re)built, its stored value is within s/2 of the value quantised."""
    cfg = _small_cfg(budget_tokens=1000, k_bits=4, v_bits=4)
    fr = _frames(cfg, 1, seed=5)
    cache = xo.OracleCache(cfg)
    q, k, v = fr[0]
    cache.step(q, k, v)
    kt = k.transpose(1, 0, 2)
    grp = np.arange(cache.cache_len) // cfg.k_group
    assert np.all(np.abs(cache.stored_k() - kt) <= 0.5 * cache.Ks[:, grp, :] * (1 + 1e-4))
    vt = v.transpose(1, 0, 2)
    assert np.all(np.abs(cache.stored_v() - vt) <= 0.5 * np.repeat(cache.Vs, cfg.v_group, axis=2) * (1 + 1e-4))


def test_value_codes_are_the_same_whether_requantised_or_carried():
    cfg_a = _small_cfg(k_bits=4, v_bits=4)
    cfg_b = _small_cfg(k_bits=4, v_bits=4, requant_v=True)
    fr = _frames(cfg_a, 8, seed=6)
    a, b = xo.OracleCache(cfg_a), xo.OracleCache(cfg_b)
    for f in fr:
        a.step(*f)
        b.step(*f)
        assert np.array_equal(a.Vc, b.Vc)
        assert np.array_equal(a.ids, b.ids)


def test_unchanged_key_groups_are_carried():
    """Groups lying wholly below the first dropped position keep their codes and
    (s, z); groups from there on are rebuilt."""
    cfg = _small_cfg(k_bits=4, v_bits=4)
    fr = _frames(cfg, 7, seed=8)
    cache = xo.OracleCache(cfg)
    G = cfg.k_group
    for f in fr:
        ids_b, Kc_b, Ks_b, Kz_b = cache.ids.copy(), cache.Kc.copy(), cache.Ks.copy(), cache.Kz.copy()
        cache.step(*f)
        if cache.last_keep is not None:
            keep = cache.last_keep
            T = len(ids_b) + cfg.tokens_per_frame
            dropped = np.setdiff1d(np.arange(T), keep)
            p0 = int(dropped.min())
            g0 = p0 // G
            assert g0 >= 1
            assert np.array_equal(cache.Kc[:, :g0 * G], Kc_b[:, :g0 * G])
            assert np.array_equal(cache.Ks[:, :g0], Ks_b[:, :g0])
            assert np.array_equal(cache.Kz[:, :g0], Kz_b[:, :g0])


def test_determinism():
    cfg = _small_cfg(k_bits=4, v_bits=4)
    fr = _frames(cfg, 6, seed=9)
    runs = []
    for _ in range(2):
        cache = xo.OracleCache(cfg)
        outs = [cache.step(*f) for f in fr]
        runs.append((outs, cache.Kc.copy(), cache.Vc.copy(), cache.ids.copy()))
    assert all(np.array_equal(x, y) for x, y in zip(runs[0][0], runs[1][0]))
    assert np.array_equal(runs[0][1], runs[1][1]) and np.array_equal(runs[0][3], runs[1][3])


def test_tiny_workload_pruning_onset():
    """The 'tiny' configuration: 69 tokens per frame, budget 256: pruning starts at the
    fourth frame (276 > 256) and drops 20 tokens; later steps drop 69."""
    w = si.WORKLOADS["tiny"]
    cfg = xo.OracleConfig(w.n_heads, w.head_dim, w.tokens_per_frame, w.n_special, w.pool_group,
                          w.budget_tokens, w.k_bits, w.k_group, w.v_bits, w.v_group)
    sigma = si.key_channel_scales(w)
    cache = xo.OracleCache(cfg)
    for t in range(w.frames):
        T_before = cache.cache_len
        out = cache.step(*si.frame_qkv(w, t, sigma=sigma))
        assert np.all(np.isfinite(out))
        if t < 3:
            assert cache.last_keep is None and cache.cache_len == 69 * (t + 1)
        else:
            assert cache.cache_len == 256
            assert T_before + 69 - 256 == (20 if t == 3 else 69)
            assert len(cache.last_scores) == T_before - 69


def test_bf16_inputs_are_representable():
    w = si.WORKLOADS["vggt_layer"]
    q, k, v = si.frame_qkv(w, 0)
    for a in (q, k, v):
        assert a.dtype == np.float32 and a.shape == (1041, 16, 64)
        assert np.all(a.view(np.uint32) & 0xFFFF == 0)
    # a few key channels dominate
    sig = si.key_channel_scales(w)
    assert sig.max() / np.median(sig) > 5


def test_kept_ids_recomputed_from_the_printed_equations():
    """Pruning only (quant off): after every pruning step the cache holds exactly the first frame, the current
    frame and the k best of the tokens in between, with the scores recomputed here from Eq. 2-6 as printed
    (pooled query per head, head means of query and key, N_pooled x M product, column means) on the true keys
    of the tokens the cache held, addressed by id."""
    cfg = _small_cfg(quant=False, budget_tokens=37)
    fr = _frames(cfg, 9, seed=21)
    n, ns, g = cfg.tokens_per_frame, cfg.n_special, cfg.pool_group
    all_k = np.concatenate([f[1] for f in fr], axis=0).astype(np.float64)      # [frames * n, H, d] by token id
    cache = xo.OracleCache(cfg)
    pruned = 0
    for t, (q, k, v) in enumerate(fr):
        ids_before = cache.ids.copy()
        cache.step(q, k, v)
        ids = np.concatenate([ids_before, t * n + np.arange(n)])
        T = len(ids)
        if T <= cfg.budget_tokens:
            assert np.array_equal(cache.ids, ids)
            continue
        pruned += 1
        q64 = q.astype(np.float64)
        rows = [q64[i] for i in range(ns)]                                       # Eq. 2: [H, d] per pooled row
        a = ns
        while a < n:
            rows.append(q64[a:min(a + g, n)].mean(axis=0))
            a += g
        q_bar = np.stack(rows).mean(axis=1)                                      # Eq. 3: [N_pooled, d]
        mid_ids = ids[n:T - n]
        k_bar = all_k[mid_ids].mean(axis=1)                                      # Eq. 4: [M, d]
        s = (q_bar @ k_bar.T).mean(axis=0)                                       # Eq. 5-6: [M]
        kk = cfg.budget_tokens - 2 * n
        order = np.argsort(-s, kind="stable")
        best = np.sort(order[:kk])
        margin = s[order[kk - 1]] - s[order[kk]]
        assert margin > 1e-4 * np.abs(s).max(), "near-tie in the test data: pick another seed"
        expect = np.concatenate([ids[:n], mid_ids[best], ids[T - n:]])
        assert np.array_equal(cache.ids, expect), f"frame {t}"
    assert pruned >= 5


def test_every_stored_key_follows_its_own_token():
    """A token's stored key moves by at most half a quantisation step of its new group whenever its group is
    rebuilt, and not at all when the group is carried: followed by token id across compaction, so codes or
    metadata left behind for a group whose members changed would show."""
    cfg = _small_cfg(k_bits=4, v_bits=4, budget_tokens=41)
    fr = _frames(cfg, 9, seed=22)
    n, G = cfg.tokens_per_frame, cfg.k_group
    cache = xo.OracleCache(cfg)
    value = {}                                   # token id -> its key as last stored, [H, d]
    for t, (q, k, v) in enumerate(fr):
        for i in range(n):
            value[t * n + i] = k[i].astype(np.float32)
        cache.step(q, k, v)
        stored = cache.stored_k()                # [H, T, d]
        grp = np.arange(cache.cache_len) // G
        step = cache.Ks[:, grp, :]
        for pos, tid in enumerate(cache.ids):
            prev = value[int(tid)]
            assert np.all(np.abs(stored[:, pos, :] - prev) <= 0.5 * step[:, pos, :] * (1 + 1e-4) + 1e-30), (t, pos, int(tid))
            value[int(tid)] = stored[:, pos, :].copy()
