"""Pins for the oracle's slot-stable cache (a surviving token never moves, freed slots take the new tokens, a key
group is re-quantised only when it receives a new member; paper Sec. 3.2 keep set, Sec. 3.3 Eq. 7-9 per group).

Expected values come from the compacting oracle (same keep sets whenever keys are held as fp32 values), from
following every token by id, and from the quantiser's own error bound."""
import numpy as np
import pytest

from oracle import xstream_oracle as xo


def _cfg(**kw):
    base = dict(n_heads=2, head_dim=16, tokens_per_frame=11, n_special=3, pool_group=4,
                budget_tokens=40, k_bits=4, k_group=8, v_bits=4, v_group=16)
    base.update(kw)
    return xo.OracleConfig(**base)


def _frames(cfg, count, seed=0):
    rng = np.random.default_rng(seed)
    sig = np.exp(rng.standard_normal((cfg.n_heads, cfg.head_dim))).astype(np.float32)
    shape = (cfg.tokens_per_frame, cfg.n_heads, cfg.head_dim)
    return [(rng.standard_normal(shape).astype(np.float32),
             (rng.standard_normal(shape).astype(np.float32) * sig).astype(np.float32),
             rng.standard_normal(shape).astype(np.float32)) for _ in range(count)]


@pytest.mark.parametrize("budget", [22, 37, 40, 64])
def test_same_tokens_and_outputs_as_the_compacting_cache_when_keys_are_values(budget):
    """Pruning only: the score of a token depends on its key and the query, not on where it is stored, so both
    layouts keep the same token set and give the same attention output at every step."""
    fr = _frames(_cfg(), 10, seed=1)
    a = xo.OracleCache(_cfg(quant=False, budget_tokens=budget, slot_stable=True))
    b = xo.OracleCache(_cfg(quant=False, budget_tokens=budget))
    for t, f in enumerate(fr):
        oa, ob = a.step(*f), b.step(*f)
        assert np.abs(oa - ob).max() < 1e-12, t
        assert sorted(a.ids.tolist()) == sorted(b.ids.tolist()), t
        # and the stored key of every token is the same value in both
        order_a, order_b = np.argsort(a.ids), np.argsort(b.ids)
        assert np.array_equal(a.K[:, order_a], b.K[:, order_b]) and np.array_equal(a.V[:, order_a], b.V[:, order_b])


@pytest.mark.parametrize("meta16", [False, True])
def test_tokens_never_move_and_untouched_groups_are_bit_identical(meta16):
    cfg = _cfg(slot_stable=True, meta16=meta16)
    n, L, G = cfg.tokens_per_frame, cfg.budget_tokens, cfg.k_group
    fr = _frames(cfg, 12, seed=2)
    cache = xo.OracleCache(cfg)
    slot_of = {}
    touched_total = untouched_total = 0
    for t, f in enumerate(fr):
        before = dict(ids=cache.ids.copy())
        if t:
            before.update(Kc=cache.Kc.copy(), Ks=cache.Ks.copy(), Kz=cache.Kz.copy(), Vc=cache.Vc.copy(), Vs=cache.Vs.copy(),
                          Vz=cache.Vz.copy(), K=cache.stored_k().copy())
        cache.step(*f)
        T = cache.cache_len
        assert T == min((t + 1) * n, L)
        assert np.array_equal(cache.ids[:n], np.arange(n))                      # the first frame keeps slots 0..n-1
        assert set(range(t * n, (t + 1) * n)) <= set(cache.ids.tolist())          # the current frame is kept
        assert len(set(cache.ids.tolist())) == T
        for slot, tok in enumerate(cache.ids.tolist()):
            assert slot_of.setdefault(tok, slot) == slot, f"token {tok} moved"
        if not t:
            continue
        T_old = len(before["ids"])
        changed = np.array([s >= T_old or before["ids"][s] != cache.ids[s] for s in range(T)])
        # the new tokens, in order, sit in the changed slots in ascending slot order
        assert np.array_equal(cache.ids[changed], t * n + np.arange(n))
        for gidx in range(-(-T // G)):
            a, b = gidx * G, min((gidx + 1) * G, T)
            if changed[a:b].any():
                touched_total += 1
                # survivors of a re-quantised group move by at most half a step of the new grid
                grp_s = cache.Ks[:, gidx][:, None, :]
                now = cache.stored_k()[:, a:b]
                for j, slot in enumerate(range(a, b)):
                    if not changed[slot]:
                        assert np.all(np.abs(now[:, j] - before["K"][:, slot]) <= 0.5 * grp_s[:, 0] * (1 + 1e-4))
            else:
                untouched_total += 1
                assert np.array_equal(cache.Kc[:, a:b], before["Kc"][:, a:b])
                assert np.array_equal(cache.Ks[:, gidx], before["Ks"][:, gidx]) and np.array_equal(cache.Kz[:, gidx], before["Kz"][:, gidx])
        keep_slots = ~changed[:T_old]
        assert np.array_equal(cache.Vc[:, :T_old][:, keep_slots], before["Vc"][:, keep_slots])
        assert np.array_equal(cache.Vs[:, :T_old][:, keep_slots], before["Vs"][:, keep_slots])
    assert touched_total > 10 and untouched_total > 10


def test_new_tokens_are_quantised_from_their_inputs():
    """A group made only of new tokens (warm-up, whole groups appended) holds Eq. 7-8 of the inputs."""
    cfg = _cfg(slot_stable=True, tokens_per_frame=16, n_special=0, budget_tokens=64)
    fr = _frames(cfg, 2, seed=3)
    cache = xo.OracleCache(cfg)
    cache.step(*fr[0])
    cache.step(*fr[1])
    k1 = fr[1][1].transpose(1, 0, 2)
    codes, s, z = xo.quantize_k_group(k1[:, :8], cfg.k_bits)
    assert np.array_equal(cache.Kc[:, 16:24], codes) and np.array_equal(cache.Ks[:, 2], s) and np.array_equal(cache.Kz[:, 2], z)


def test_dropped_tokens_are_the_lowest_scored_of_the_stored_keys():
    """With codes: the tokens that lose their slot are exactly the lowest of the scores the step exported, and
    last_keep lists the surviving slots in ascending order followed by the new tokens."""
    cfg = _cfg(slot_stable=True)
    n, L = cfg.tokens_per_frame, cfg.budget_tokens
    fr = _frames(cfg, 9, seed=4)
    cache = xo.OracleCache(cfg)
    pruned = 0
    for t, f in enumerate(fr):
        ids_before = cache.ids.copy()
        cache.step(*f)
        T_old = len(ids_before)
        if T_old + n <= L:
            assert cache.last_keep is None
            continue
        pruned += 1
        scores = cache.last_scores.astype(np.float64)          # slots n .. T_old - 1
        n_drop = T_old + n - L
        order = np.argsort(scores, kind="stable")
        assert scores[order[n_drop]] - scores[order[n_drop - 1]] > 0, "tie at the cut in the test data"
        dropped = np.sort(order[:n_drop]) + n
        gone = np.array([s for s in range(T_old) if ids_before[s] != cache.ids[s]])
        assert np.array_equal(gone, dropped)
        expect_keep = np.concatenate([np.setdiff1d(np.arange(T_old), dropped), T_old + np.arange(n)])
        assert np.array_equal(cache.last_keep, expect_keep)
    assert pruned >= 5


def test_attention_reads_what_the_slots_store():
    cfg = _cfg(slot_stable=True, k_bits=8, v_bits=8)
    fr = _frames(cfg, 7, seed=5)
    cache = xo.OracleCache(cfg)
    for q, k, v in fr:
        k_old, v_old = cache.stored_k().copy(), cache.stored_v().copy()
        out = cache.step(q, k, v)
        ref = xo.attention_fp64(q, np.concatenate([k_old, k.transpose(1, 0, 2)], axis=1),
                                np.concatenate([v_old, v.transpose(1, 0, 2)], axis=1), 0.25)
        assert np.abs(out - ref).max() < 1e-12


def test_chunks_and_update_first_order_work_on_slots():
    cfg = _cfg(slot_stable=True, budget_tokens=58)
    fr = _frames(cfg, 9, seed=6)
    cache = xo.OracleCache(cfg)
    for t in range(0, 9, 3):
        q, k, v = (np.concatenate([f[j] for f in fr[t:t + 3]], axis=0) for j in range(3))
        cache.step(q, k, v)
        assert cache.cache_len == min((t + 3) * 11, 58) and len(set(cache.ids.tolist())) == cache.cache_len
        assert set(range(t * 11, (t + 3) * 11)) <= set(cache.ids.tolist())
    cfg2 = _cfg(slot_stable=True, attend_after_prune=True)
    c2 = xo.OracleCache(cfg2)
    for q, k, v in fr:
        out = c2.step(q, k, v)
        assert np.abs(out - xo.attention_fp64(q, c2.stored_k(), c2.stored_v(), 0.25)).max() < 1e-12


def test_fidelity_against_uncompressed_attention_is_no_worse_than_the_compacting_cache():
    """Both layouts against un-pruned, un-quantised attention over a long stream: keeping survivors in place must
    not cost accuracy (on stationary random streams the two are on a par: nearly every group loses a member per
    step in either layout)."""
    cfg_s = _cfg(slot_stable=True, budget_tokens=80, k_group=16)
    cfg_c = _cfg(budget_tokens=80, k_group=16)
    fr = _frames(cfg_s, 60, seed=7)
    a, b = xo.OracleCache(cfg_s), xo.OracleCache(cfg_c)
    ea = eb = 0.0
    for t, f in enumerate(fr):
        oa, ob = a.step(*f), b.step(*f)
        if t >= 30:
            ref = xo.reference_full_attention(fr, t, 0.25)
            ea += float(np.abs(oa - ref).mean())
            eb += float(np.abs(ob - ref).mean())
    assert ea <= 1.15 * eb, (ea, eb)
