"""CPU oracle for the compressed-KV streaming attention step of XStreamVGGT.

TEST INFRASTRUCTURE ONLY.  This is a plain, slow numpy implementation of what
the paper defines, written to be checked against the paper by eye.  It shares
no code with the HIP path and must never be imported by the product package;
only tests, the smoke check and the benchmark's cpu_baseline leg call it.

What it follows (paper section / equation, equations counted in order of
appearance):
  * temporal attention over [cache, current frame]            Sec. 3.1, Eq. 1
  * pooled query (specials kept, patches group-averaged)      Sec. 3.2, Eq. 2
  * head-mean of the pooled query                             Sec. 3.2, Eq. 3
  * head-mean of the prunable (middle) keys                   Sec. 3.2, Eq. 4
  * score matrix and its mean over pooled queries             Sec. 3.2, Eq. 5-6
  * top-k, k = max(0, L_max - T_first - T_current), keep set  Sec. 3.2
  * asymmetric uniform quantiser                              Sec. 3.3, Eq. 7-8
  * per-channel keys / per-token values                       Sec. 3.3, Eq. 9
  * dequantisation at attention time                          Sec. 3.3, Eq. 10

Precision: attention is evaluated in fp64.  Everything that decides an integer
(the importance scores that feed top-k, the quantiser's scale, zero-point and
codes) is evaluated in fp32 with one rounding per arithmetic operation and a
fixed order of additions, stated at each function, because the kept indices and
the codes are compared bit-for-bit.  The paper gives no evaluation order for
Eq. 5-6; the one fixed here for keys held as codes (importance_scores_codes)
pulls the per-group factors q~ s and -z q~ s out of the per-token work.

Readings of points the paper leaves open (each also listed in the design
notes): attention runs before pruning and the current frame enters its own
attention at input precision (the attend_after_prune switch takes the other
order: update first, attend over codes only); a call may carry a chunk of
several frames, attended with the frame-wise causal mask and appended as one
block of current tokens; a short last patch group is averaged over its
own size; ties in top-k keep the lower cache position and survivors stay in
ascending position order (the slot_stable switch keeps every survivor in its
slot instead and fills the freed slots with the new tokens); rounding is to nearest-even; the zero-point is not
clamped (with 16-bit metadata, the meta16 switch, scales are rounded up to their
storage format before anything is computed from them and zero-points are kept
to 12 bits); a quantisation group is re-quantised only when its ordered member
list changed (so value groups, one token each, are quantised once); a short
trailing key group is quantised over the tokens present; a constant group gets
scale |min| (1 if min is 0).

Pins (tests/test_oracle_*.py): brute-force attention in pure Python loops,
the literal Eq. 2-6 matrix form in fp64, closed-form quantiser cases and a
hand-worked fixture, a full-sort top-k, and whole-step invariants.
Task-level accuracy (paper Tables 1-4) is parity unpinned: it needs datasets
and trained weights that are not available.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

F32 = np.float32


@dataclass
class OracleConfig:
    n_heads: int
    head_dim: int
    tokens_per_frame: int            # n
    n_special: int                   # camera + register tokens, first in the frame
    pool_group: int                  # g
    budget_tokens: int               # L_max
    k_bits: int = 4
    k_group: int = 64                # tokens per per-channel key group
    v_bits: int = 4
    v_group: int = 64                # channels per per-token value group
    softmax_scale: float = 0.0       # 0 -> 1/sqrt(head_dim)
    quant: bool = True               # False: keep fp32 K/V (pruning only)
    requant_v: bool = False          # True: re-quantise V every step (literal reading; diagnostic)
    meta16: bool = False             # True: 16-bit scales and zero-points (see quant_params_meta16_k / _v)
    slot_stable: bool = False        # True: tokens never move: a pruned token frees its slot and the new tokens fill the
                                     #       freed slots in ascending order (no compaction); a key group is the 64 (k_group)
                                     #       consecutive slots and is re-quantised only when it receives a new member
    attend_after_prune: bool = False # True: the other reading of Fig. 2's order: append, prune, quantise, then attend
                                     #       over the compressed cache (current frame in codes, exactly <= L_max keys)


# --------------------------------------------------------------------------
# Quantiser, Sec. 3.3 Eq. 7-8.
# --------------------------------------------------------------------------
def quant_params(mn: np.ndarray, mx: np.ndarray, bits: int):
    """Scale and zero-point of Eq. 8 from a group's min and max, in fp32.

    s = (max - min) / (2^b - 1);  z = round(-min / s), ties to even.
    A constant group (max == min) has no defined scale in the paper; it gets
    s = |min| (1 if min == 0), which reconstructs it exactly with code 0.
    """
    mn = np.asarray(mn, dtype=F32)
    mx = np.asarray(mx, dtype=F32)
    levels = F32(2 ** bits - 1)
    s = ((mx - mn) / levels).astype(F32)
    flat = mx == mn
    if np.any(flat):
        alt = np.where(mn != 0, np.abs(mn), F32(1)).astype(F32)
        s = np.where(flat, alt, s).astype(F32)
    z = np.rint((-mn) / s).astype(np.int32)
    return s, z


# 16-bit metadata (the storage the paper's quantiser, KIVI with INT4 and group 64 in its
# experimental setup, keeps its scales in).  A scale that is rounded for storage has to be
# rounded *up*, and before the zero-point and the codes are computed from it, or the group's
# maximum would leave the code range and the s/2 error bound of Eq. 7-8 would break.
META16_S_MIN = F32(2.0 ** -14)       # smallest normal half
META16_S_MAX = F32(2048.0)
META16_Z_MIN, META16_Z_MAX = -1024, 1023


def round_up_sig_bits(x: np.ndarray, bits: int) -> np.ndarray:
    """Smallest fp32 value >= x (x > 0, finite) that has at most `bits` significant bits."""
    u = np.ascontiguousarray(x, dtype=F32).view(np.uint32).astype(np.uint64)
    mask = np.uint64((1 << (24 - bits)) - 1)
    up = (u | mask) + np.uint64(1)
    return np.where((u & mask) != 0, up, u).astype(np.uint32).view(F32).reshape(np.shape(x))


def logit_scale_log2(softmax_scale: float) -> np.float32:
    """softmax scale times log2(e) as one fp32 product: the factor that takes q . k to the
    base-2 logit of Eq. 1's softmax."""
    return F32(F32(softmax_scale) * F32(1.4426950408889634))


def quant_params_meta16_k(mn: np.ndarray, mx: np.ndarray, bits: int, c_log2: np.float32):
    """Eq. 8 for a key group with 16-bit metadata.

    What is stored is the scale in the logit domain, a = s * c_log2 (the step of one code in
    the base-2 logit per unit of query), rounded up to 7 significant bits and kept inside the
    half range [2^-14, 2048]: with 7 bits, a * (code - z) is exact in an 11-bit significand for
    |code - z| <= 16, so the de-quantised key enters Eq. 1 without a further rounding.  The
    scale that Eq. 7 / Eq. 10 use is s = a * (1 / c_log2), the reciprocal rounded to fp32 once
    and one fp32 multiply per scale (every consumer of a stored scale re-derives s, so it is a
    multiply rather than a divide).  The zero-point is kept in [-1024, 1023] (12 bits, exact
    beside a code in a half).  Returns (a, s, z).
    """
    mn = np.asarray(mn, dtype=F32)
    s_raw, _ = quant_params(mn, mx, bits)
    a_raw = (s_raw * c_log2).astype(F32)
    a = np.clip(round_up_sig_bits(a_raw, 7), META16_S_MIN, META16_S_MAX).astype(F32)
    inv_c = F32(F32(1.0) / c_log2)
    s = (a * inv_c).astype(F32)
    z = np.clip(np.rint((-mn) / s), META16_Z_MIN, META16_Z_MAX).astype(np.int32)
    return a, s, z


def quant_params_meta16_v(mn: np.ndarray, mx: np.ndarray, bits: int):
    """Eq. 8 for a value group with 16-bit metadata: s rounded up to a half (11 significant
    bits) inside [2^-14, 2048], z in [-1024, 1023].  Returns (s, z)."""
    mn = np.asarray(mn, dtype=F32)
    s_raw, _ = quant_params(mn, mx, bits)
    s = np.clip(round_up_sig_bits(s_raw, 11), META16_S_MIN, META16_S_MAX).astype(F32)
    z = np.clip(np.rint((-mn) / s), META16_Z_MIN, META16_Z_MAX).astype(np.int32)
    return s, z


def quant_codes(x: np.ndarray, s: np.ndarray, z: np.ndarray, bits: int) -> np.ndarray:
    """Eq. 7: clamp(round(x / s) + z, 0, 2^b - 1); fp32 divide, ties to even."""
    x = np.asarray(x, dtype=F32)
    r = np.rint(x / s.astype(F32)).astype(np.int64) + z.astype(np.int64)
    return np.clip(r, 0, 2 ** bits - 1).astype(np.uint8)


def dequant(codes: np.ndarray, s: np.ndarray, z: np.ndarray) -> np.ndarray:
    """Eq. 10: x~ = s * (code - z), the difference formed exactly, one fp32 multiply."""
    diff = (codes.astype(np.int64) - z.astype(np.int64)).astype(F32)
    return (s.astype(F32) * diff).astype(F32)


def quantize_k_group(xg: np.ndarray, bits: int, meta16_c_log2=None):
    """Per-channel key quantisation (Eq. 9) of one group.

    xg: fp32 [H, m, d], m <= k_group tokens.  One (s, z) per (head, channel),
    taken over the m tokens.  meta16_c_log2: None for fp32 metadata, else the
    logit factor of quant_params_meta16_k.
    """
    mn = xg.min(axis=1)
    mx = xg.max(axis=1)
    if meta16_c_log2 is None:
        s, z = quant_params(mn, mx, bits)
    else:
        _, s, z = quant_params_meta16_k(mn, mx, bits, meta16_c_log2)
    codes = quant_codes(xg, s[:, None, :], z[:, None, :], bits)
    return codes, s, z


def quantize_v_tokens(xv: np.ndarray, bits: int, v_group: int, meta16: bool = False):
    """Per-token value quantisation (Eq. 9).

    xv: fp32 [H, m, d].  One (s, z) per (head, token, group of v_group channels).
    Returns codes [H, m, d], s and z [H, m, d // v_group].
    """
    H, m, d = xv.shape
    ng = d // v_group
    xr = xv.reshape(H, m, ng, v_group)
    mn = xr.min(axis=3)
    mx = xr.max(axis=3)
    s, z = quant_params_meta16_v(mn, mx, bits) if meta16 else quant_params(mn, mx, bits)
    codes = quant_codes(xr, s[..., None], z[..., None], bits).reshape(H, m, d)
    return codes, s, z


# --------------------------------------------------------------------------
# Attention, Sec. 3.1 Eq. 1 (fp64).
# --------------------------------------------------------------------------
def attention_fp64(q: np.ndarray, k_all: np.ndarray, v_all: np.ndarray, scale: float) -> np.ndarray:
    """softmax(q k^T * scale) v per head.

    q [n, H, d]; k_all, v_all [H, T, d].  Returns fp64 [n, H, d].  Every query
    of the frame sees every cached token and every token of its own frame
    (frame-wise causal attention with one frame per step has no masked entry).
    """
    n, H, d = q.shape
    out = np.empty((n, H, d), dtype=np.float64)
    for h in range(H):
        qh = q[:, h, :].astype(np.float64)
        kh = k_all[h].astype(np.float64)
        vh = v_all[h].astype(np.float64)
        logits = (qh @ kh.T) * float(scale)
        logits -= logits.max(axis=1, keepdims=True)
        p = np.exp(logits)
        p /= p.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ vh
    return out


# --------------------------------------------------------------------------
# Importance score, Sec. 3.2 Eq. 2-6.
# --------------------------------------------------------------------------
def pooled_groups(n: int, n_special: int, g: int):
    """Row ranges of the pooled query (Eq. 2): each special token alone, then
    consecutive patch-token groups of g; a short last group keeps its own size."""
    groups = [(i, i + 1) for i in range(n_special)]
    a = n_special
    while a < n:
        groups.append((a, min(a + g, n)))
        a += g
    return groups


def pooled_query_mean(q: np.ndarray, n_special: int, g: int, n_frame: int = 0) -> np.ndarray:
    """q~[c] = mean over pooled rows of the head-mean pooled query (Eq. 2-3 and
    the row-mean of Eq. 6 pulled inside the product), in fp32.

    Order of operations (one rounding each):
      per (head, pooled row): add the group's tokens in ascending order, divide by its size;
      per pooled row: add heads 0..H-1 in order, divide by H;
      add pooled rows in ascending order, divide by N_pooled.

    n_frame: tokens per frame when q holds several frames one after the other (a chunk):
    every frame is pooled by itself (its special tokens, then its patch groups) and the
    rows of all frames are averaged together, in frame order.  0: q is one frame.
    """
    q = np.asarray(q, dtype=F32)
    n, H, d = q.shape
    if n_frame and n_frame != n:
        assert n % n_frame == 0
        groups = [(f * n_frame + a, f * n_frame + b) for f in range(n // n_frame) for (a, b) in pooled_groups(n_frame, n_special, g)]
    else:
        groups = pooled_groups(n, n_special, g)
    acc_rows = np.zeros(d, dtype=F32)
    for (a, b) in groups:
        acc_h = np.zeros(d, dtype=F32)
        for h in range(H):
            acc = q[a, h, :].copy()
            for t in range(a + 1, b):
                acc = (acc + q[t, h, :]).astype(F32)
            pooled = (acc / F32(b - a)).astype(F32)
            acc_h = (acc_h + pooled).astype(F32)
        qbar = (acc_h / F32(H)).astype(F32)
        acc_rows = (acc_rows + qbar).astype(F32)
    return (acc_rows / F32(len(groups))).astype(F32)


def tree_dot(qt: np.ndarray, kd: np.ndarray) -> np.ndarray:
    """Dot products q~ . kd[..., :] in fp32 with a fixed pairwise order.

    p[c] = q~[c] * kd[..., c]; then for m = d/2, d/4, ..., 1: p[c] += p[c + m]
    for c < m.  Result p[0].  d must be a power of two.
    """
    p = (qt.astype(F32) * kd.astype(F32)).astype(F32)
    m = p.shape[-1] // 2
    while m >= 1:
        p = (p[..., :m] + p[..., m:2 * m]).astype(F32)
        m //= 2
    return p[..., 0]


def importance_scores(qt: np.ndarray, k_mid: np.ndarray) -> np.ndarray:
    """S_j of Eq. 6 for the middle tokens, in fp32.

    Eq. 5-6 average the rows of Qbar Kbar^T; by linearity that is q~ . Kbar_j
    with q~ the row-mean of Qbar, and Kbar_j the head-mean key (Eq. 4).
    Evaluated as: per head D[h, j] = tree_dot(q~, K[h, j, :]); then add heads
    0..H-1 in order and divide by H.

    k_mid: fp32 [H, M, d].  This is the form for keys held as fp32 values (the
    pruning-only cache); keys held as codes go through importance_scores_codes.
    """
    H = k_mid.shape[0]
    D = tree_dot(qt, k_mid)                       # [H, M]
    acc = D[0].copy()
    for h in range(1, H):
        acc = (acc + D[h]).astype(F32)
    return (acc / F32(H)).astype(F32)


def fma32(x: np.ndarray, y: np.ndarray, z: np.ndarray) -> np.ndarray:
    """x * y + z with one rounding to fp32 (a fused multiply-add), for fp32 inputs.

    Evaluated in fp64: the product of two fp32 values is exact there, and the sum is exact
    whenever the two terms' exponents are within 20 of each other or one of them is zero,
    which holds for every use below unless a zero-point exceeds 2^20 (such groups are
    reported as range warnings; for them the last bit of a score may differ from a true
    fused operation with probability around 2^-29 per term).
    """
    return (x.astype(np.float64) * y.astype(np.float64) + z.astype(np.float64)).astype(F32)


def importance_scores_codes(qt: np.ndarray, codes: np.ndarray, s: np.ndarray, z: np.ndarray, grp: np.ndarray) -> np.ndarray:
    """S_j of Eq. 6 for middle tokens held as codes, in fp32.

    The same quantity as importance_scores (q~ . Kbar_j with the keys of Eq. 10), with the
    per-group constants pulled out of the per-token work: per head, key group and channel
    a = q~[c] * s[c] and b = -float(z[c]) * a (one rounding each); per token and channel
    p[c] = fma(float(code[c]), a[c], b[c]) (one rounding); then the same stride-halving tree
    over the channels, heads added 0..H-1 in order, divided by H.

    codes: uint8 [H, M, d]; s fp32 and z int32 [H, G, d]; grp: int [M], key group of each token.
    """
    H = codes.shape[0]
    a = (qt.astype(F32)[None, None, :] * s.astype(F32)).astype(F32)                  # [H, G, d]
    b = ((-z.astype(F32)) * a).astype(F32)
    p = fma32(codes.astype(F32), a[:, grp, :], b[:, grp, :])                          # [H, M, d]
    m = p.shape[-1] // 2
    while m >= 1:
        p = (p[..., :m] + p[..., m:2 * m]).astype(F32)
        m //= 2
    D = p[..., 0]
    acc = D[0].copy()
    for h in range(1, H):
        acc = (acc + D[h]).astype(F32)
    return (acc / F32(H)).astype(F32)


def importance_scores_literal(q: np.ndarray, k_mid: np.ndarray, n_special: int, g: int) -> np.ndarray:
    """Eq. 2-6 exactly as printed, matrix form, in fp64 (used only as a pin)."""
    q = q.astype(np.float64)
    n, H, d = q.shape
    groups = pooled_groups(n, n_special, g)
    q_pooled = np.stack([q[a:b].mean(axis=0) for (a, b) in groups], axis=1)   # [H, N_pooled, d]
    q_bar = q_pooled.mean(axis=0)                                             # Eq. 3
    k_bar = k_mid.astype(np.float64).mean(axis=0)                             # Eq. 4  [M, d]
    s_matrix = q_bar @ k_bar.T                                                # Eq. 5
    return s_matrix.mean(axis=0)                                              # Eq. 6


def order_key(s: np.ndarray) -> np.ndarray:
    """Monotone uint32 image of fp32 values (total order; -0.0 below +0.0)."""
    u = np.ascontiguousarray(s, dtype=F32).view(np.uint32)
    neg = (u >> 31).astype(bool)
    return np.where(neg, ~u, u | np.uint32(0x80000000)).astype(np.uint32)


def select_keep(scores: np.ndarray, T: int, n_first: int, n_current: int, budget: int) -> np.ndarray:
    """Keep set of Sec. 3.2: first frame, top-k of the middle, current frame.

    scores: fp32 [T - n_first - n_current] for cache positions n_first ..
    T - n_current - 1.  k = max(0, budget - n_first - n_current).  Among equal
    scores the lower position is kept.  Returns ascending positions.
    """
    M = T - n_first - n_current
    assert scores.shape == (M,)
    k = max(0, budget - n_first - n_current)
    k = min(k, M)
    key = order_key(scores).astype(np.int64)
    pos = np.arange(M, dtype=np.int64)
    # descending key, then ascending position
    order = np.lexsort((pos, -key))
    mid = np.sort(order[:k]) + n_first
    return np.concatenate([np.arange(n_first), mid, np.arange(T - n_current, T)]).astype(np.int32)


# --------------------------------------------------------------------------
# The streaming cache.
# --------------------------------------------------------------------------
class OracleCache:
    """One (stream, layer) cache; step() is one frame of the hot path."""

    def __init__(self, cfg: OracleConfig):
        self.cfg = cfg
        H, d = cfg.n_heads, cfg.head_dim
        assert d % cfg.v_group == 0
        self.frames = 0
        self.ids = np.zeros(0, dtype=np.int32)
        if cfg.quant:
            self.Kc = np.zeros((H, 0, d), dtype=np.uint8)
            self.Ks = np.zeros((H, 0, d), dtype=F32)
            self.Kz = np.zeros((H, 0, d), dtype=np.int32)
            self.Vc = np.zeros((H, 0, d), dtype=np.uint8)
            self.Vs = np.zeros((H, 0, d // cfg.v_group), dtype=F32)
            self.Vz = np.zeros((H, 0, d // cfg.v_group), dtype=np.int32)
        else:
            self.K = np.zeros((H, 0, d), dtype=F32)
            self.V = np.zeros((H, 0, d), dtype=F32)
        self.last_keep = None
        self.last_scores = None
        self.k_groups_requantised = 0

    # -- views of the stored cache -------------------------------------------------
    @property
    def cache_len(self) -> int:
        return int(self.ids.shape[0])

    def stored_k(self) -> np.ndarray:
        c = self.cfg
        if not c.quant:
            return self.K
        grp = np.arange(self.cache_len) // c.k_group
        return dequant(self.Kc, self.Ks[:, grp, :], self.Kz[:, grp, :])

    def stored_v(self) -> np.ndarray:
        c = self.cfg
        if not c.quant:
            return self.V
        s = np.repeat(self.Vs, c.v_group, axis=2)
        z = np.repeat(self.Vz, c.v_group, axis=2)
        return dequant(self.Vc, s, z)

    # -- one frame, or a chunk of frames ----------------------------------------------
    def step(self, q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
        """One call of the hot path.  q, k, v: [F n, H, d], F >= 1 consecutive frames.

        Frame-wise causal attention (Sec. 3.1, Eq. 1): a query of the chunk's frame a sees the
        cache as it was before the call and the chunk's frames 0..a at input precision.  The
        cache is then updated once with the whole chunk as the current tokens: T_current = F n,
        k = max(0, L_max - T_first - T_current), the pooled query of Eq. 2-3 taken over all F
        frames.  With attend_after_prune the update comes first and attention runs over the
        updated cache (one frame per call in that order).
        """
        c = self.cfg
        m, H, d = q.shape
        n = c.tokens_per_frame
        assert (H, d) == (c.n_heads, c.head_dim) and m >= n and m % n == 0
        F = m // n
        assert not (c.attend_after_prune and F > 1)
        q = np.asarray(q, dtype=F32)
        k_new = np.ascontiguousarray(np.asarray(k, dtype=F32).transpose(1, 0, 2))   # [H, F n, d]
        v_new = np.ascontiguousarray(np.asarray(v, dtype=F32).transpose(1, 0, 2))
        scale = c.softmax_scale if c.softmax_scale != 0 else 1.0 / np.sqrt(d)

        # Eq. 10 then Eq. 1: de-quantise the cache, attend over [cache; the chunk up to the query's frame].
        k_old = self.stored_k()
        v_old = self.stored_v()
        k_all = np.concatenate([k_old, k_new], axis=1)
        v_all = np.concatenate([v_old, v_new], axis=1)
        T_old = self.cache_len
        out = None
        if not c.attend_after_prune:
            out = np.empty((m, H, d), dtype=np.float64)
            for a in range(F):
                hi = T_old + (a + 1) * n
                out[a * n:(a + 1) * n] = attention_fp64(q[a * n:(a + 1) * n], k_all[:, :hi, :], v_all[:, :hi, :], scale)

        # Append (Sec. 3.1, last sentence).
        ids_all = np.concatenate([self.ids, self.frames * n + np.arange(m, dtype=np.int32)]).astype(np.int32)
        T = T_old + m
        old_ids = self.ids

        # Prune when the cache length exceeds the budget (Sec. 3.2).
        self.last_keep = None
        self.last_scores = None
        if T > c.budget_tokens:
            n_first = min(n, T_old)          # tokens of the first frame (when it is not part of this very chunk)
            n_current = m
            qt = pooled_query_mean(q, c.n_special, c.pool_group, n)
            if c.quant:
                # the middle tokens are all cached (the current tokens are the last n_current positions)
                pos = np.arange(n_first, T - n_current)
                scores = importance_scores_codes(qt, self.Kc[:, pos, :], self.Ks, self.Kz, pos // c.k_group)
            else:
                scores = importance_scores(qt, k_all[:, n_first:T - n_current, :])
            keep = select_keep(scores, T, n_first, n_current, c.budget_tokens)
            self.last_keep = keep
            self.last_scores = scores
        else:
            keep = np.arange(T, dtype=np.int32)

        if c.slot_stable:
            self._update_slots(keep, T_old, m, ids_all, k_all, k_new, v_new, scale)
            self.frames += F
            if c.attend_after_prune:
                out = attention_fp64(q, self.stored_k(), self.stored_v(), scale)
            return out

        ids_new = ids_all[keep]
        k_fin = k_all[:, keep, :]
        T_fin = keep.shape[0]

        if not c.quant:
            self.K = k_fin
            self.V = v_all[:, keep, :]
            self.ids = ids_new
            self.frames += F
            if c.attend_after_prune:
                out = attention_fp64(q, self.K, self.V, scale)
            return out

        # Values: quantised once when their frame is appended, then carried (their
        # one-token groups never change membership).
        vc_new, vs_new, vz_new = quantize_v_tokens(v_new, c.v_bits, c.v_group, c.meta16)
        if c.requant_v:
            v_fin = v_all[:, keep, :]
            Vc, Vs, Vz = quantize_v_tokens(v_fin, c.v_bits, c.v_group, c.meta16)
        else:
            Vc = np.concatenate([self.Vc, vc_new], axis=1)[:, keep, :]
            Vs = np.concatenate([self.Vs, vs_new], axis=1)[:, keep, :]
            Vz = np.concatenate([self.Vz, vz_new], axis=1)[:, keep, :]

        # Keys: groups of k_group consecutive cache positions; a group whose ordered
        # member list is unchanged is carried, every other group is re-quantised from
        # the fp32 values of its members (de-quantised old tokens, input new tokens).
        G = c.k_group
        n_groups = (T_fin + G - 1) // G
        Kc = np.zeros((H, T_fin, d), dtype=np.uint8)
        Ks = np.zeros((H, n_groups, d), dtype=F32)
        Kz = np.zeros((H, n_groups, d), dtype=np.int32)
        for m in range(n_groups):
            a, b = m * G, min((m + 1) * G, T_fin)
            old_a, old_b = m * G, min((m + 1) * G, T_old)
            same = (old_b - old_a == b - a) and np.array_equal(old_ids[old_a:old_b], ids_new[a:b])
            if same:
                Kc[:, a:b, :] = self.Kc[:, a:b, :]
                Ks[:, m, :] = self.Ks[:, m, :]
                Kz[:, m, :] = self.Kz[:, m, :]
            else:
                codes, s, z = quantize_k_group(k_fin[:, a:b, :], c.k_bits, logit_scale_log2(scale) if c.meta16 else None)
                Kc[:, a:b, :] = codes
                Ks[:, m, :] = s
                Kz[:, m, :] = z
                self.k_groups_requantised += 1

        self.Kc, self.Ks, self.Kz = Kc, Ks, Kz
        self.Vc, self.Vs, self.Vz = Vc, Vs, Vz
        self.ids = ids_new
        self.frames += F
        if c.attend_after_prune:
            # Eq. 1 over the compressed cache: every key, the current frame's included, is a de-quantised code
            out = attention_fp64(q, self.stored_k(), self.stored_v(), scale)
        return out


def _update_slots(self, keep, T_old, m, ids_all, k_all, k_new, v_new, scale):
    """Slot-stable cache update (the drift-reducing storage of Sec. 3.3's "quantization is applied to the
    final KV cache" read per group): which tokens survive is the keep set of Sec. 3.2 exactly as in the
    compacting cache; where they live is not.  A surviving token stays in its slot.  The free slots, the
    dropped tokens' slots in ascending order followed by the never-used tail [T_old, L_max), receive the
    call's new tokens in order.  Values, one group per token, are written once.  A key group (k_group
    consecutive slots) that received no new member keeps its codes, scale and zero-point bit for bit;
    one that did is re-quantised by Eq. 7-8 over its present members (stored values of the survivors,
    inputs of the new tokens)."""
    c = self.cfg
    L, G = c.budget_tokens, c.k_group
    kept_old = keep[keep < T_old]
    if keep.shape[0] < T_old + m:                      # pruned: some cached slots are freed
        occupied = np.zeros(T_old, dtype=bool)
        occupied[kept_old] = True
        free = np.concatenate([np.flatnonzero(~occupied), np.arange(T_old, max(L, T_old))])
    else:
        free = np.arange(T_old, T_old + m)
    assign = free[:m].astype(np.int64)                  # slot of the call's i-th new token
    assert assign.shape[0] == m, "the budget must hold the first frame and the call's tokens"
    T_new = max(T_old, int(assign.max()) + 1)
    new_ids = ids_all[T_old:]

    def grown(a, fill=0):
        out = np.full(a.shape[:1] + (T_new,) + a.shape[2:], fill, dtype=a.dtype) if a.ndim > 1 else np.full((T_new,), fill, dtype=a.dtype)
        if a.ndim > 1:
            out[:, :a.shape[1]] = a
        else:
            out[:a.shape[0]] = a
        return out

    ids = grown(self.ids)
    ids[assign] = new_ids
    if not c.quant:
        K, V = grown(self.K), grown(self.V)
        K[:, assign] = k_new
        V[:, assign] = v_new
        self.K, self.V, self.ids = K, V, ids
        return
    vc_new, vs_new, vz_new = quantize_v_tokens(v_new, c.v_bits, c.v_group, c.meta16)
    Vc, Vs, Vz = grown(self.Vc), grown(self.Vs), grown(self.Vz)
    Vc[:, assign], Vs[:, assign], Vz[:, assign] = vc_new, vs_new, vz_new
    k_old = self.stored_k()                             # Eq. 10 of every slot as stored before the call
    n_groups = (T_new + G - 1) // G
    H, d = c.n_heads, c.head_dim
    Kc = grown(self.Kc)
    Ks = np.zeros((H, n_groups, d), dtype=F32)
    Kz = np.zeros((H, n_groups, d), dtype=np.int32)
    Ks[:, :self.Ks.shape[1]] = self.Ks
    Kz[:, :self.Kz.shape[1]] = self.Kz
    slot_token = np.full(T_new, -1, dtype=np.int64)     # index of the new token a slot receives, or -1
    slot_token[assign] = np.arange(m)
    for gidx in np.unique(assign // G):
        a, b = gidx * G, min((gidx + 1) * G, T_new)
        vals = np.empty((H, b - a, d), dtype=F32)
        for j, slot in enumerate(range(a, b)):
            vals[:, j] = k_new[:, slot_token[slot]] if slot_token[slot] >= 0 else k_old[:, slot]
        codes, s_, z_ = quantize_k_group(vals, c.k_bits, logit_scale_log2(scale) if c.meta16 else None)
        Kc[:, a:b], Ks[:, gidx], Kz[:, gidx] = codes, s_, z_
        self.k_groups_requantised += 1
    self.Kc, self.Ks, self.Kz = Kc, Ks, Kz
    self.Vc, self.Vs, self.Vz = Vc, Vs, Vz
    self.ids = ids


OracleCache._update_slots = _update_slots


def reference_full_attention(frames_qkv, upto: int, scale: float) -> np.ndarray:
    """Un-pruned, un-quantised Eq. 1 for frame `upto` (0-based) over all earlier
    frames plus its own: the quantity the compressed step approximates."""
    q = frames_qkv[upto][0]
    k_all = np.concatenate([np.asarray(f[1], dtype=F32).transpose(1, 0, 2) for f in frames_qkv[:upto + 1]], axis=1)
    v_all = np.concatenate([np.asarray(f[2], dtype=F32).transpose(1, 0, 2) for f in frames_qkv[:upto + 1]], axis=1)
    return attention_fp64(np.asarray(q, dtype=F32), k_all, v_all, scale)
