"""Pins for the oracle's attention (Eq. 1), importance score (Eq. 2-6) and top-k keep set."""
import math

import numpy as np
import pytest

from oracle import xstream_oracle as xo


# ----------------------------------------------------------------------------- attention
def _brute_attention(q, k_all, v_all, scale):
    """Pure-Python softmax attention, one scalar at a time."""
    n, H, d = q.shape
    T = k_all.shape[1]
    out = [[[0.0] * d for _ in range(H)] for _ in range(n)]
    for i in range(n):
        for h in range(H):
            logits = [scale * sum(float(q[i, h, c]) * float(k_all[h, j, c]) for c in range(d)) for j in range(T)]
            mx = max(logits)
            w = [math.exp(l - mx) for l in logits]
            tot = sum(w)
            for c in range(d):
                out[i][h][c] = sum(w[j] * float(v_all[h, j, c]) for j in range(T)) / tot
    return np.array(out)


def test_attention_matches_pure_python_brute_force():
    rng = np.random.default_rng(0)
    n, H, d, T = 5, 2, 8, 13
    q = rng.standard_normal((n, H, d)).astype(np.float32)
    k = rng.standard_normal((H, T, d)).astype(np.float32) * 2
    v = rng.standard_normal((H, T, d)).astype(np.float32)
    got = xo.attention_fp64(q, k, v, 0.37)
    exp = _brute_attention(q, k, v, 0.37)
    assert np.abs(got - exp).max() < 1e-12


def test_attention_invariants():
    rng = np.random.default_rng(1)
    n, H, d, T = 7, 3, 16, 40
    q = rng.standard_normal((n, H, d)).astype(np.float32)
    k = rng.standard_normal((H, T, d)).astype(np.float32)
    v = rng.standard_normal((H, T, d)).astype(np.float32)
    out = xo.attention_fp64(q, k, v, 0.25)
    # convex combination of value rows, per head and channel
    for h in range(H):
        assert np.all(out[:, h, :] <= v[h].max(axis=0) + 1e-12)
        assert np.all(out[:, h, :] >= v[h].min(axis=0) - 1e-12)
    # the order of cached tokens does not matter
    perm = rng.permutation(T)
    out_p = xo.attention_fp64(q, k[:, perm], v[:, perm], 0.25)
    assert np.abs(out - out_p).max() < 1e-12
    # a single key: the output is that key's value whatever the query
    one = xo.attention_fp64(q, k[:, :1], v[:, :1], 0.25)
    assert np.abs(one - v[:, 0, :][None]).max() < 1e-12
    # scale 0: uniform weights -> mean of values
    uni = xo.attention_fp64(q, k, v, 0.0)
    assert np.abs(uni - v.astype(np.float64).mean(axis=1)[None]).max() < 1e-12


# ----------------------------------------------------------------------------- score
def _brute_scores(q, k_mid, n_special, g):
    """Eq. 2-6 with explicit loops in Python floats."""
    n, H, d = q.shape
    M = k_mid.shape[1]
    rows = [(i, i + 1) for i in range(n_special)]
    a = n_special
    while a < n:
        rows.append((a, min(a + g, n)))
        a += g
    qbar = []
    for (a, b) in rows:                                      # Eq. 2 then Eq. 3
        vec = [0.0] * d
        for h in range(H):
            for c in range(d):
                vec[c] += sum(float(q[t, h, c]) for t in range(a, b)) / (b - a) / H
        qbar.append(vec)
    kbar = [[sum(float(k_mid[h, j, c]) for h in range(H)) / H for c in range(d)] for j in range(M)]   # Eq. 4
    s = []
    for j in range(M):                                       # Eq. 5-6
        s.append(sum(sum(qbar[i][c] * kbar[j][c] for c in range(d)) for i in range(len(rows))) / len(rows))
    return np.array(s), len(rows)


@pytest.mark.parametrize("n,n_special,g", [(21, 5, 4), (22, 5, 4), (9, 1, 16), (6, 0, 1)])
def test_scores_match_brute_force_and_literal(n, n_special, g):
    rng = np.random.default_rng(n)
    H, d, M = 3, 8, 17
    q = rng.standard_normal((n, H, d)).astype(np.float32)
    k_mid = (rng.standard_normal((H, M, d)) * np.exp(rng.standard_normal((H, 1, d)))).astype(np.float32)
    qt = xo.pooled_query_mean(q, n_special, g)
    got = xo.importance_scores(qt, k_mid).astype(np.float64)
    brute, n_rows = _brute_scores(q, k_mid, n_special, g)
    assert n_rows == len(xo.pooled_groups(n, n_special, g)) == n_special + -(-(n - n_special) // g)
    lit = xo.importance_scores_literal(q, k_mid, n_special, g)
    tol = 1e-5 * np.abs(brute).max() + 1e-7
    assert np.abs(lit - brute).max() < 1e-12
    assert np.abs(got - brute).max() < tol


def test_scores_textbook_special_case():
    """g = 1, one head: S_j = mean_i q_i . k_j."""
    rng = np.random.default_rng(5)
    n, d, M = 6, 16, 9
    q = rng.standard_normal((n, 1, d)).astype(np.float32)
    k = rng.standard_normal((1, M, d)).astype(np.float32)
    qt = xo.pooled_query_mean(q, 2, 1)
    s = xo.importance_scores(qt, k)
    exp = (q[:, 0, :].astype(np.float64) @ k[0].astype(np.float64).T).mean(axis=0)
    assert np.abs(s - exp).max() < 1e-5


def test_tree_dot_order():
    """The pairwise order is the stride-halving one: with values chosen so that
    fp32 addition is not associative, only that order gives the expected bits."""
    d = 8
    qt = np.ones(d, dtype=np.float32)
    big = np.float32(2.0 ** 24)
    kd = np.array([big, 1, 1, 1, -big, 1, 1, 1], dtype=np.float32)
    # level 1 pairs (c, c+4): (big-big)=0, 2, 2, 2 ; level 2 pairs (c, c+2): 2, 4 ; level 3: 6
    assert float(xo.tree_dot(qt, kd)) == 6.0
    # a left-to-right sum would give: big+1+1+1 = big (absorbed), -big -> 0, +3 -> 3
    seq = np.float32(0)
    for x in kd:
        seq = np.float32(seq + x)
    assert float(seq) == 3.0


def test_score_scaling_keeps_the_kept_set():
    rng = np.random.default_rng(9)
    n, H, d, M = 21, 2, 16, 50
    q = rng.standard_normal((n, H, d)).astype(np.float32)
    k = rng.standard_normal((H, M, d)).astype(np.float32)
    s1 = xo.importance_scores(xo.pooled_query_mean(q, 5, 4), k)
    s2 = xo.importance_scores(xo.pooled_query_mean(q * np.float32(4), 5, 4), k)
    assert np.array_equal(s2, s1 * np.float32(4))          # powers of two scale exactly
    T = M + 2 * n
    assert np.array_equal(xo.select_keep(s1, T, n, n, 2 * n + 20), xo.select_keep(s2, T, n, n, 2 * n + 20))


# ----------------------------------------------------------------------------- top-k
def _brute_keep(scores, T, n_first, n_cur, budget):
    M = len(scores)
    k = min(max(0, budget - n_first - n_cur), M)
    left = list(range(M))

    def better(a, b):     # is a strictly preferred to b
        sa, sb = float(scores[a]), float(scores[b])
        if sa != sb:
            return sa > sb
        za, zb = math.copysign(1, sa), math.copysign(1, sb)
        if sa == 0 and za != zb:
            return za > zb
        return a < b
    chosen = []
    for _ in range(k):
        best = left[0]
        for c in left[1:]:
            if better(c, best):
                best = c
        chosen.append(best)
        left.remove(best)
    return list(range(n_first)) + sorted(c + n_first for c in chosen) + list(range(T - n_cur, T))


@pytest.mark.parametrize("seed", range(6))
def test_keep_set_matches_brute_force(seed):
    rng = np.random.default_rng(seed)
    n = 7
    M = int(rng.integers(1, 40))
    T = M + 2 * n
    budget = int(rng.integers(2 * n, T + 3))
    scores = rng.standard_normal(M).astype(np.float32)
    if seed % 2:
        scores = np.round(scores * 2) / 2                    # many exact ties
        scores[rng.integers(0, M)] = -0.0
    scores = scores.astype(np.float32)
    got = xo.select_keep(scores, T, n, n, budget)
    assert got.tolist() == _brute_keep(scores, T, n, n, budget)
    assert len(got) == min(T, max(budget, 2 * n))
    assert np.all(np.diff(got) > 0)


def test_keep_ties_prefer_lower_position_and_budget_below_two_frames():
    n = 3
    scores = np.array([1, 2, 2, 2, 0], dtype=np.float32)
    T = 5 + 2 * n
    got = xo.select_keep(scores, T, n, n, 2 * n + 2)
    assert got.tolist() == [0, 1, 2, 4, 5, 8, 9, 10]
    # k = max(0, budget - first - current) = 0: only first and current frames survive
    got0 = xo.select_keep(scores, T, n, n, n)
    assert got0.tolist() == [0, 1, 2, 8, 9, 10]


def test_order_key_is_monotone():
    vals = np.array([-np.inf, -3.5, -1e-30, -0.0, 0.0, 1e-30, 2.0, np.inf], dtype=np.float32)
    keys = xo.order_key(vals).astype(np.int64)
    assert np.all(np.diff(keys) > 0)


# ----------------------------------------------------------------------------- score over codes
def _quantised_keys(rng, H, M, d, bits, G):
    k = (rng.standard_normal((H, M, d)) * np.exp(rng.standard_normal((H, 1, d)))).astype(np.float32)
    ng = -(-M // G)
    codes = np.zeros((H, M, d), np.uint8)
    s = np.zeros((H, ng, d), np.float32)
    z = np.zeros((H, ng, d), np.int32)
    for m in range(ng):
        c_, s_, z_ = xo.quantize_k_group(k[:, m * G:(m + 1) * G, :], bits)
        codes[:, m * G:(m + 1) * G, :], s[:, m], z[:, m] = c_, s_, z_
    return codes, s, z, np.arange(M) // G


@pytest.mark.parametrize("bits,G", [(4, 8), (2, 4), (8, 16)])
def test_scores_over_codes_match_the_printed_equations(bits, G):
    """The code form against Eq. 2-6 as printed (fp64, brute force) on the de-quantised keys."""
    rng = np.random.default_rng(bits)
    n, H, d, M, n_special, g = 21, 3, 8, 29, 5, 4
    q = rng.standard_normal((n, H, d)).astype(np.float32)
    codes, s, z, grp = _quantised_keys(rng, H, M, d, bits, G)
    k_deq = xo.dequant(codes, s[:, grp, :], z[:, grp, :])
    qt = xo.pooled_query_mean(q, n_special, g)
    got = xo.importance_scores_codes(qt, codes, s, z, grp).astype(np.float64)
    brute, _ = _brute_scores(q, k_deq, n_special, g)
    assert np.abs(got - brute).max() < 1e-5 * np.abs(brute).max() + 1e-7
    # and within the same band of the value form, whose kept set it must share away from near-ties
    other = xo.importance_scores(qt, k_deq).astype(np.float64)
    assert np.abs(got - other).max() < 1e-5 * np.abs(brute).max() + 1e-7


def _round_fraction_to_f32(fr):
    """Correctly rounded (nearest, ties to even) fp32 value of an exact rational, by integer arithmetic."""
    from fractions import Fraction
    if fr == 0:
        return np.float32(0.0)
    sign = -1 if fr < 0 else 1
    fr = abs(fr)
    e = 0
    while fr >= 2 ** 24:
        fr /= 2
        e += 1
    while fr < 2 ** 23:
        fr *= 2
        e -= 1
    n, rem = divmod(fr.numerator, fr.denominator)
    twice = 2 * rem
    if twice > fr.denominator or (twice == fr.denominator and n % 2 == 1):
        n += 1
    return np.float32(sign * float(Fraction(n) * Fraction(2) ** e))


def test_fused_multiply_add_is_a_single_rounding():
    """fma32 against exact rational arithmetic rounded once, on code x scale + offset shaped operands
    (including sums that land next to an fp32 tie)."""
    from fractions import Fraction
    rng = np.random.default_rng(17)
    code = rng.integers(0, 256, size=3000).astype(np.float32)
    a = (rng.standard_normal(3000) * np.exp(rng.normal(0, 3, 3000))).astype(np.float32)
    zf = rng.integers(-300, 300, size=3000).astype(np.float32)
    b = (-zf * a).astype(np.float32)
    got = xo.fma32(code, a, b)
    for i in range(3000):
        exact = Fraction(float(code[i])) * Fraction(float(a[i])) + Fraction(float(b[i]))
        assert got[i] == _round_fraction_to_f32(exact), i
    # a product that needs more than 24 bits, where rounding the product first would differ
    x, y, zc = np.float32(3.0), np.float32(1 + 2.0 ** -23), np.float32(-3.0)
    assert xo.fma32(x, y, zc) == np.float32(3 * 2.0 ** -23)
    assert np.float32(np.float32(x * y) + zc) != np.float32(3 * 2.0 ** -23)


def test_scores_over_codes_follow_the_stated_order():
    """One head, one group, hand-sized: a = q~ s, b = -z a, p = fma(code, a, b), then the stride-halving tree."""
    d = 4
    qt = np.array([1.0, 2.0, 0.5, 1.0], np.float32)
    s = np.array([[[0.5, 0.25, 2.0, 1.0]]], np.float32)
    z = np.array([[[1, 0, 2, 3]]], np.int32)
    codes = np.array([[[3, 4, 1, 3], [0, 0, 0, 0]]], np.uint8)
    # a = [0.5, 0.5, 1, 1], b = [-0.5, 0, -2, -3]; token 0: p = [1, 2, -1, 0] -> (1 + -1) + (2 + 0) = 2; token 1: p = b -> -5.5
    got = xo.importance_scores_codes(qt, codes, s, z, np.array([0, 0]))
    assert got.tolist() == [2.0, -5.5]
    # equals q~ . (s (code - z)) exactly here
    kd = xo.dequant(codes, s[:, [0, 0], :], z[:, [0, 0], :])
    assert xo.importance_scores(qt, kd).tolist() == [2.0, -5.5]
