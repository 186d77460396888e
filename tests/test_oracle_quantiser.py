"""Pins for the oracle's quantiser (paper Sec. 3.3, Eq. 7-10).

None of these re-type the oracle's formula in numpy: expected values come from
a hand-worked fixture, from exact rational arithmetic, from closed forms, or
from the error bound the scheme guarantees.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import xstream_oracle as xo

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "quantiser_cases.txt")


def _cases():
    out = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            bits, xs, s, z, codes = [p.strip() for p in line.split("|")]
            out.append((int(bits), [float(t) for t in xs.split()], float(s), int(z), [int(t) for t in codes.split()]))
    return out


@pytest.mark.parametrize("bits,xs,s_exp,z_exp,codes_exp", _cases())
def test_hand_worked_fixture(bits, xs, s_exp, z_exp, codes_exp):
    x = np.array(xs, dtype=np.float32)
    s, z = xo.quant_params(x.min(), x.max(), bits)
    assert float(s) == s_exp and int(z) == z_exp
    codes = xo.quant_codes(x, s, z, bits)
    assert codes.tolist() == codes_exp


def _round_half_even(fr: Fraction) -> int:
    return round(fr)          # Python rounds Fractions to nearest, ties to even


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_exact_rational_arithmetic(bits, seed):
    """Dyadic inputs make every fp32 operation exact, so Eq. 7-8 can be evaluated
    with Fractions (including ties) and must match bit for bit."""
    rng = np.random.default_rng(seed)
    levels = 2 ** bits - 1
    for _ in range(50):
        kexp = int(rng.integers(-6, 4))
        step = Fraction(2) ** kexp                      # the scale, a power of two
        lo = Fraction(int(rng.integers(-4 * levels, 4 * levels)), 8) * step
        hi = lo + levels * step
        m = int(rng.integers(2, 70))
        offs = rng.integers(0, 8 * levels + 1, size=m)  # multiples of step / 8: exact halves appear
        xs = [lo + Fraction(int(o), 8) * step for o in offs]
        xs[0], xs[-1] = lo, hi
        x = np.array([float(v) for v in xs], dtype=np.float32)
        assert all(Fraction(float(a)) == b for a, b in zip(x, xs))
        s, z = xo.quant_params(x.min(), x.max(), bits)
        assert Fraction(float(s)) == step
        z_exp = _round_half_even(-lo / step)
        assert int(z) == z_exp
        codes = xo.quant_codes(x, s, z, bits)
        exp = [min(max(_round_half_even(v / step) + z_exp, 0), levels) for v in xs]
        assert codes.tolist() == exp
        back = xo.dequant(codes, s, z)
        exp_back = [float(step * (c - z_exp)) for c in exp]
        assert back.tolist() == exp_back


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_integer_ramp_is_identity(bits):
    levels = 2 ** bits - 1
    x = np.arange(levels + 1, dtype=np.float32)
    s, z = xo.quant_params(x.min(), x.max(), bits)
    assert float(s) == 1.0 and int(z) == 0
    codes = xo.quant_codes(x, s, z, bits)
    assert np.array_equal(codes, x.astype(np.uint8))
    assert np.array_equal(xo.dequant(codes, s, z), x)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_error_bound_and_extremes(bits):
    """|x - DQ(Q(x))| <= s/2 (up to fp32 rounding of s); min -> code 0."""
    rng = np.random.default_rng(bits)
    levels = 2 ** bits - 1
    for _ in range(200):
        m = int(rng.integers(2, 65))
        x = (rng.standard_normal(m) * np.exp(rng.standard_normal()) + rng.standard_normal()).astype(np.float32)
        s, z = xo.quant_params(x.min(), x.max(), bits)
        codes = xo.quant_codes(x, s, z, bits)
        assert codes.min() >= 0 and codes.max() <= levels
        assert codes[np.argmin(x)] == 0
        assert codes[np.argmax(x)] >= levels - 1
        back = xo.dequant(codes, s, z).astype(np.float64)
        err = np.abs(back - x.astype(np.float64))
        assert err.max() <= 0.5 * float(s) * (1 + 1e-4) + 1e-6 * float(s) * (abs(int(z)) + levels)


def test_constant_group():
    for val in [3.0, -2.5, 0.0]:
        x = np.full(5, val, dtype=np.float32)
        s, z = xo.quant_params(x.min(), x.max(), 4)
        codes = xo.quant_codes(x, s, z, 4)
        assert np.all(codes == 0)
        assert np.array_equal(xo.dequant(codes, s, z), x)


def test_requantising_untouched_group_is_idempotent():
    """De-quantise -> quantise of the same group reproduces the codes (the
    basis for carrying value codes and unchanged key groups)."""
    rng = np.random.default_rng(7)
    bad = 0
    for _ in range(300):
        x = rng.standard_normal(64).astype(np.float32) * np.float32(np.exp(rng.standard_normal()))
        s, z = xo.quant_params(x.min(), x.max(), 4)
        c = xo.quant_codes(x, s, z, 4)
        y = xo.dequant(c, s, z)
        s2, z2 = xo.quant_params(y.min(), y.max(), 4)
        c2 = xo.quant_codes(y, s2, z2, 4)
        bad += int(not np.array_equal(c, c2))
    assert bad == 0


def test_per_channel_keys_beat_per_token_keys():
    """Paper Sec. 3.3: with a few dominant key channels, per-channel groups give a
    much smaller error than per-token groups."""
    rng = np.random.default_rng(3)
    H, m, d = 2, 64, 64
    sigma = np.exp(rng.standard_normal((H, 1, d)) * 1.5).astype(np.float32)
    k = (rng.standard_normal((H, m, d)).astype(np.float32) * sigma)
    codes, s, z = xo.quantize_k_group(k, 4)
    err_channel = np.abs(xo.dequant(codes, s[:, None, :], z[:, None, :]) - k).mean()
    codes_t, st, zt = xo.quantize_v_tokens(k, 4, 64)
    back_t = xo.dequant(codes_t, np.repeat(st, 64, axis=2), np.repeat(zt, 64, axis=2))
    err_token = np.abs(back_t - k).mean()
    assert err_channel < 0.5 * err_token


def test_group_axes():
    """Keys: one (s, z) per (head, channel) over tokens; values: one per (head, token, channel group)."""
    rng = np.random.default_rng(11)
    x = rng.standard_normal((3, 10, 64)).astype(np.float32)
    codes, s, z = xo.quantize_k_group(x, 4)
    assert s.shape == (3, 64) and z.shape == (3, 64) and codes.shape == x.shape
    # every (head, channel) column reaches code 0 at its own minimum
    assert np.all(np.take_along_axis(codes, x.argmin(axis=1)[:, None, :], axis=1) == 0)
    codes_v, sv, zv = xo.quantize_v_tokens(x, 4, 32)
    assert sv.shape == (3, 10, 2)
    xr = x.reshape(3, 10, 2, 32)
    cr = codes_v.reshape(3, 10, 2, 32)
    assert np.all(np.take_along_axis(cr, xr.argmin(axis=3)[..., None], axis=3) == 0)
