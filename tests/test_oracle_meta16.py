"""Pins for the oracle's 16-bit-metadata quantiser variant (paper Sec. 3.3, Eq. 7-10 with the
scale and zero-point held in 16 bits each).

Expected values come from a hand-worked fixture, from exact rational arithmetic, from the half
type of numpy used as an independent rounding device, and from the properties the variant is
built to have (range still covered, error bound of Eq. 7-8, exact products in a half).
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import xstream_oracle as xo

F32 = np.float32
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "meta16_scale_cases.txt")


def _cases():
    out = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            bits, x, exp = [p.strip() for p in line.split("|")][:3]
            out.append((int(bits), int(x, 16), int(exp, 16)))
    return out


@pytest.mark.parametrize("bits,x_hex,exp_hex", _cases())
def test_round_up_hand_worked(bits, x_hex, exp_hex):
    x = np.array([x_hex], dtype=np.uint32).view(F32)
    got = xo.round_up_sig_bits(x, bits).view(np.uint32)[0]
    assert int(got) == exp_hex


def _ceil_sig(x: float, bits: int) -> Fraction:
    """Exact: x = m 2^e with m in [1/2, 1); round m up to a multiple of 2^-bits."""
    m, e = math.frexp(x)
    fm = Fraction(m) * 2 ** bits
    return Fraction(math.ceil(fm), 2 ** bits) * Fraction(2) ** e


@pytest.mark.parametrize("bits", [7, 11])
def test_round_up_against_exact_arithmetic(bits):
    rng = np.random.default_rng(5)
    x = np.exp(rng.normal(0, 4, size=4000)).astype(F32)
    got = xo.round_up_sig_bits(x, bits)
    for a, b in zip(x.tolist(), got.tolist()):
        assert Fraction(b) == _ceil_sig(a, bits)


def test_round_up_to_11_bits_is_the_next_half():
    """numpy's half as an independent device: nearest half, moved up one when it fell below."""
    rng = np.random.default_rng(6)
    x = np.exp(rng.normal(0, 2, size=4000)).astype(F32)          # inside the normal half range
    h = x.astype(np.float16)
    h = np.where(h.astype(F32) < x, np.nextafter(h, np.float16(np.inf)), h)
    assert np.array_equal(xo.round_up_sig_bits(x, 11), h.astype(F32))


@pytest.mark.parametrize("bits", [2, 4])
def test_key_products_are_exact_in_a_half(bits):
    """The stored logit-domain scale has 7 significant bits, so a * (code - z) fits the 11-bit
    significand of a half whenever |code - z| <= 16: converting the fp32 product to half and back
    changes nothing."""
    rng = np.random.default_rng(7)
    c = xo.logit_scale_log2(0.125)
    x = (rng.standard_normal((500, 64)) * np.exp(rng.normal(0, 1, size=(500, 1)))).astype(F32)
    a, s, z = xo.quant_params_meta16_k(x.min(axis=1), x.max(axis=1), bits, c)
    assert np.all((z >= 0) & (z <= 2 ** bits - 1))               # zero-mean groups straddle zero
    codes = xo.quant_codes(x, s[:, None], z[:, None], bits).astype(np.int64)
    m = (codes - z[:, None]).astype(F32)
    prod = (a[:, None] * m).astype(F32)
    assert np.array_equal(prod.astype(np.float16).astype(F32), prod)
    # and a itself is a half with at most 7 significant bits
    assert np.array_equal(a.astype(np.float16).astype(F32), a)
    assert np.all((a.view(np.uint32) & np.uint32(0x1FFFF)) == 0)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_scale_only_ever_grows_and_by_little(bits):
    rng = np.random.default_rng(8)
    c = xo.logit_scale_log2(0.125)
    mn = -np.exp(rng.normal(0, 1, size=2000)).astype(F32)
    mx = np.exp(rng.normal(0, 1, size=2000)).astype(F32)
    s_raw, _ = xo.quant_params(mn, mx, bits)
    a, s, z = xo.quant_params_meta16_k(mn, mx, bits, c)
    r = s.astype(np.float64) / s_raw.astype(np.float64)
    assert np.all(r >= 1 - 2e-7) and np.all(r <= 1 + 2.0 ** -6 + 2e-7)
    sv, zv = xo.quant_params_meta16_v(mn, mx, bits)
    rv = sv.astype(np.float64) / s_raw.astype(np.float64)
    assert np.all(rv >= 1.0) and np.all(rv <= 1 + 2.0 ** -10)


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("which", ["k", "v"])
def test_error_bound_and_extremes_survive_the_rounded_scale(bits, which):
    """|x - s (code - z)| <= s / 2 (up to fp32 rounding of the quotient), the group minimum
    still maps to code 0, and the maximum to a code within the 2^-6 (keys) or 2^-10 (values)
    that the scale may have grown, so the top of the code range is still used."""
    rng = np.random.default_rng(9)
    c = xo.logit_scale_log2(0.125)
    x = (rng.standard_normal((300, 64)) * np.exp(rng.normal(0, 1.5, size=(300, 1)))).astype(F32)
    mn, mx = x.min(axis=1), x.max(axis=1)
    if which == "k":
        _, s, z = xo.quant_params_meta16_k(mn, mx, bits, c)
    else:
        s, z = xo.quant_params_meta16_v(mn, mx, bits)
    codes = xo.quant_codes(x, s[:, None], z[:, None], bits)
    back = xo.dequant(codes, s[:, None], z[:, None])
    err = np.abs(back.astype(np.float64) - x)
    assert np.all(err <= 0.5 * s[:, None].astype(np.float64) * (1 + 1e-5))
    lo = codes[np.arange(300), x.argmin(axis=1)]
    hi = codes[np.arange(300), x.argmax(axis=1)]
    assert np.all(lo == 0)
    levels = 2 ** bits - 1
    grow = 2.0 ** -6 if which == "k" else 2.0 ** -10
    assert np.all(hi >= levels / (1 + grow) - 1) and np.all(hi <= levels)


def test_saturation_of_scale_and_zero_point():
    c = xo.logit_scale_log2(0.125)
    # a group far from zero: -min / s would be 100000, kept at 1023; one far above: -1024
    a, s, z = xo.quant_params_meta16_k(np.array([-100000.0], F32), np.array([-99985.0], F32), 4, c)
    assert z[0] == 1023
    a, s, z = xo.quant_params_meta16_k(np.array([100000.0], F32), np.array([100015.0], F32), 4, c)
    assert z[0] == -1024
    # scales beyond the half range
    a, s, z = xo.quant_params_meta16_k(np.array([-1e-9], F32), np.array([1e-9], F32), 4, c)
    assert a[0] == F32(2.0 ** -14)
    a, s, z = xo.quant_params_meta16_k(np.array([-1e6], F32), np.array([1e6], F32), 4, c)
    assert a[0] == F32(2048.0)
    sv, zv = xo.quant_params_meta16_v(np.array([-1e-9], F32), np.array([1e-9], F32), 4)
    assert sv[0] == F32(2.0 ** -14)
    sv, zv = xo.quant_params_meta16_v(np.array([-1e6], F32), np.array([1e6], F32), 4)
    assert sv[0] == F32(2048.0)


def test_scale_follows_the_softmax_scale():
    """The stored key scale is a logit-domain quantity: with another softmax scale the same group
    gets another grid point, and s = a * (1 / c) always reproduces from what is stored."""
    mn, mx = np.array([-1.3], F32), np.array([2.1], F32)
    for scale in (0.125, 0.1, 1.0):
        c = xo.logit_scale_log2(scale)
        a, s, z = xo.quant_params_meta16_k(mn, mx, 4, c)
        assert s[0] == F32(a[0] * F32(F32(1.0) / c))
        assert abs(float(s[0]) * float(c) / float(a[0]) - 1) < 3e-7
        assert Fraction(float(a[0])) == _ceil_sig(float(F32(F32((mx[0] - mn[0]) / F32(15)) * c)), 7)


def _stream(cfg, frames, seed):
    rng = np.random.default_rng(seed)
    H, d, n = cfg.n_heads, cfg.head_dim, cfg.tokens_per_frame
    sigma = np.exp(rng.standard_normal((H, d))).astype(F32)
    out = []
    for _ in range(frames):
        q = rng.standard_normal((n, H, d)).astype(F32)
        k = (rng.standard_normal((n, H, d)) * sigma).astype(F32)
        v = rng.standard_normal((n, H, d)).astype(F32)
        out.append((q, k, v))
    return out


@pytest.mark.parametrize("k_bits,k_group,v_bits,v_group", [(4, 64, 4, 64), (2, 32, 4, 32), (8, 64, 8, 64)])
def test_whole_step_invariants_with_16_bit_metadata(k_bits, k_group, v_bits, v_group):
    cfg = xo.OracleConfig(2, 64, 37, 5, 16, 150, k_bits, k_group, v_bits, v_group, meta16=True)
    cache = xo.OracleCache(cfg)
    c = xo.logit_scale_log2(0.125)
    prev = None
    for t, (q, k, v) in enumerate(_stream(cfg, 9, 3)):
        cache.step(q, k, v)
        assert cache.cache_len == min((t + 1) * 37, 150)
        # what is stored is representable in the 16-bit formats
        a = (cache.Ks * c).astype(F32)
        a7 = xo.round_up_sig_bits(a, 7)
        assert np.all(np.abs(a7.astype(np.float64) / a - 1) < 2.0 ** -6)       # s = a / c came from a 7-bit a
        assert np.array_equal(cache.Vs.astype(np.float16).astype(F32), cache.Vs)
        assert cache.Kz.min() >= -1024 and cache.Kz.max() <= 1023
        # a key group whose members did not change is carried bit for bit
        if prev is not None and cache.last_keep is not None:
            p0 = int(np.flatnonzero(cache.last_keep != np.arange(len(cache.last_keep)))[0]) if np.any(
                cache.last_keep != np.arange(len(cache.last_keep))) else len(cache.last_keep)
            g_keep = p0 // k_group
            assert np.array_equal(cache.Kc[:, :g_keep * k_group], prev[0][:, :g_keep * k_group])
            assert np.array_equal(cache.Ks[:, :g_keep], prev[1][:, :g_keep])
        prev = (cache.Kc.copy(), cache.Ks.copy())


def test_eight_bit_codes_with_16_bit_metadata_stay_close_to_full_attention():
    """The rounded-up scales cost at most 2^-6 of resolution: the output error against un-pruned,
    un-quantised attention stays inside the bound the fp32-metadata cache is held to, and within a
    quarter of that cache's own error."""
    cfg16 = xo.OracleConfig(2, 64, 37, 5, 16, 10 ** 6, 8, 64, 8, 64, meta16=True)
    cfg32 = xo.OracleConfig(2, 64, 37, 5, 16, 10 ** 6, 8, 64, 8, 64)
    c16, c32 = xo.OracleCache(cfg16), xo.OracleCache(cfg32)
    frames = _stream(cfg16, 5, 4)
    w16 = w32 = 0.0
    for t, (q, k, v) in enumerate(frames):
        ref = xo.reference_full_attention(frames, t, 0.125)
        w16 = max(w16, np.abs(c16.step(q, k, v) - ref).max())
        w32 = max(w32, np.abs(c32.step(q, k, v) - ref).max())
    assert w16 < 0.05 and w16 < 1.25 * w32
