"""Pins for the oracle's MXFP4 encoder/decoder (paper Eq. 2).  CPU only."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import mxfp4

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "mxfp4_worked_groups.txt")
GRID = [Fraction(0), Fraction(1, 2), Fraction(1), Fraction(3, 2), Fraction(2), Fraction(3), Fraction(4), Fraction(6)]


# ---- an independent, exact-rational statement of Eq. 2 (argmin of the distance) ----
def brute_group(vals):
    fr = [Fraction(float(v)) for v in vals]
    amax = max(abs(f) for f in fr)
    if amax == 0:
        e = -127
    else:
        k = 0
        while Fraction(2) ** k > amax:
            k -= 1
        while Fraction(2) ** (k + 1) <= amax:
            k += 1
        e = max(-127, min(127, k - 2))
    s = Fraction(2) ** e
    codes = []
    for v, f in zip(vals, fr):
        q = abs(f) / s
        best = min(range(8), key=lambda c: (abs(q - GRID[c]), c & 1))  # nearest; tie -> even code
        codes.append(best | (8 if np.signbit(np.float32(v)) else 0))
    return e + 127, codes


def oracle_group(vals):
    y = np.asarray(vals, dtype=np.float32).reshape(1, -1)
    c, s = mxfp4.quantize(y)
    return int(s[0, 0]), list(mxfp4.unpack_codes(c)[0])


def _parse_golden():
    cases = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        parts = [p.strip() for p in line.split(";")]
        name = parts[0]
        vals = [float(v) for v in parts[1].split(",")]
        fill_in, fill_out = 0.0, 0.0
        rest = parts[2:]
        if rest[0].startswith("fill="):
            fill_in = float(rest[0][5:])
            rest = rest[1:]
        byte = int(rest[0])
        exp = [float(v) for v in rest[1].split(",")]
        if len(rest) > 2 and rest[2].startswith("fill="):
            fill_out = float(rest[2][5:])
        x = np.full(32, fill_in, dtype=np.float32)
        x[:len(vals)] = vals
        d = np.full(32, fill_out, dtype=np.float64)
        d[:len(exp)] = exp
        cases.append((name, x, byte, d))
    return cases


@pytest.mark.parametrize("name,x,byte,expect", _parse_golden(), ids=[c[0] for c in _parse_golden()])
def test_hand_worked_groups(name, x, byte, expect):
    c, s = mxfp4.quantize(x.reshape(1, 32))
    assert int(s[0, 0]) == byte
    d = mxfp4.dequantize(c, s)[0]
    np.testing.assert_array_equal(d, expect)
    np.testing.assert_array_equal(np.signbit(d), np.signbit(expect))


def test_code_table_and_nibble_order():
    # one group holding magnitudes 0..7 in order at scale 1 (a 6 is present): codes are 0..7
    x = np.zeros((1, 32), dtype=np.float32)
    x[0, :8] = [0, 0.5, 1, 1.5, 2, 3, 4, 6]
    x[0, 8:16] = [-0.0, -0.5, -1, -1.5, -2, -3, -4, -6]
    c, s = mxfp4.quantize(x)
    assert s[0, 0] == 127
    # element 2i in the low nibble, 2i+1 in the high nibble
    assert list(c[0, :8]) == [0x10, 0x32, 0x54, 0x76, 0x98, 0xBA, 0xDC, 0xFE]
    assert list(mxfp4.unpack_codes(c)[0, :16]) == list(range(16))
    np.testing.assert_array_equal(mxfp4.dequantize(c, s)[0, :16], x[0, :16].astype(np.float64))


def test_scale_is_floor_log2_minus_2():
    # closed form: amax = m * 2^k with m in [1, 2)  ->  byte = k - 2 + 127
    for k in range(-120, 120, 7):
        for m in (1.0, 1.0000001, 1.5, 1.9999999):
            x = np.zeros((1, 32), dtype=np.float32)
            x[0, 5] = -np.float32(m) * np.float32(2.0) ** k
            _, s = mxfp4.quantize(x)
            assert int(s[0, 0]) == k - 2 + 127, (k, m)


def test_scale_clamps_and_zero_group():
    x = np.zeros((1, 64), dtype=np.float32)
    x[0, 0] = np.float32(2.0) ** -130         # floor(log2) - 2 = -132 -> clamp -127 -> byte 0
    x[0, 32] = np.float32(2.0) ** -126        # -128 -> clamp -127; 2^-126 / 2^-127 = 2 -> code 4
    c, s = mxfp4.quantize(x)
    assert list(s[0]) == [0, 0]
    u = mxfp4.unpack_codes(c)[0]
    assert u[0] == 0 and u[32] == 4
    assert mxfp4.dequantize(c, s)[0, 32] == 2.0 ** -126
    big = np.zeros((1, 32), dtype=np.float32)
    big[0, 0] = np.finfo(np.float32).max      # floor(log2) = 127 -> e = 125 -> byte 252 (0xFF never made)
    c, s = mxfp4.quantize(big)
    assert int(s[0, 0]) == 252 and mxfp4.unpack_codes(c)[0, 0] == 7


def test_against_exact_rational_argmin_near_every_threshold():
    """Threshold table vs. argmin-of-distance in exact rationals, on every fp32 value within
    a few ulp of each rounding boundary, at several scales, both signs."""
    ths = [0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 6.0, 7.0, 7.9999995]
    for e in (-127, -126, -20, 0, 3, 120):
        for th in ths:
            pts = [np.float32(th)]
            up = dn = np.float32(th)
            for _ in range(3):
                up = np.nextafter(up, np.float32(np.inf), dtype=np.float32)
                dn = np.nextafter(dn, np.float32(-np.inf), dtype=np.float32)
                pts += [up, dn]
            for sgn in (1.0, -1.0):
                if th < 4.0:
                    # a 4.0 pins the scale exponent at e; the points under test share its group
                    g = np.zeros(32, dtype=np.float64)
                    g[0] = 4.0
                    g[1:1 + len(pts)] = sgn * np.asarray(pts, dtype=np.float64)
                    g = np.ldexp(g, e).astype(np.float32)
                    assert oracle_group(g) == brute_group(g), (e, th, sgn)
                else:
                    # the group maximum itself is under test: one value per group
                    for p in pts:
                        g = np.zeros(32, dtype=np.float32)
                        g[3] = np.float32(np.ldexp(sgn * float(p), e))
                        assert oracle_group(g) == brute_group(g), (e, th, p)


def test_against_exact_rational_argmin_random():
    rng = np.random.default_rng(1234)
    for trial in range(300):
        kind = trial % 4
        if kind == 0:
            g = rng.standard_normal(32)
        elif kind == 1:
            g = rng.standard_normal(32) * 10.0 ** rng.uniform(-30, 30)
        elif kind == 2:
            g = rng.standard_normal(32)
            g[rng.integers(32)] *= 1000.0
        else:
            g = np.ldexp(rng.integers(-12, 13, 32) / 2.0, int(rng.integers(-10, 10)))   # many exact ties
        g = g.astype(np.float32)
        assert oracle_group(g) == brute_group(g), trial


def test_all_bf16_magnitudes_at_unit_scale():
    """Every bf16 value in [0, 8) next to a 4.0 (scale exponent 0) against the rational argmin,
    vectorised: distances are exact in fp64 because v has at most 8 significant bits."""
    bits = np.arange(0, 0x4100, dtype=np.uint32)              # 0 .. 8.0 (exclusive of 8: 0x4100 = 8.0)
    v = (bits << 16).view(np.float32)
    v = v[v < 4.0]                                            # keep amax = 4 so that e = 0
    pad = (-len(v)) % 31
    v = np.concatenate([v, np.zeros(pad, dtype=np.float32)])
    groups = np.concatenate([np.full((len(v) // 31, 1), 4.0, dtype=np.float32), v.reshape(-1, 31)], axis=1)
    c, s = mxfp4.quantize(groups)
    assert np.all(s == 127)
    got = mxfp4.unpack_codes(c)
    grid = np.array([0, 0.5, 1, 1.5, 2, 3, 4, 6])
    d = np.abs(groups.astype(np.float64)[..., None] - grid)
    # distances are exact, so equal distances are exact ties: a tiny parity penalty breaks them to the even code
    best = np.argmin(d + (np.arange(8) & 1) * 1e-12, axis=-1)
    np.testing.assert_array_equal(got & 7, best)


def test_round_trip_of_representable_inputs_and_idempotence():
    rng = np.random.default_rng(7)
    rows, G = 16, 8
    codes = rng.integers(0, 16, size=(rows, G * 32)).astype(np.uint8)
    codes[:, ::32] = rng.choice([6, 7, 14, 15], size=(rows, G))   # a 4 or a 6 in every group holds the scale
    packed = (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8)
    scales = rng.integers(90, 170, size=(rows, G)).astype(np.uint8)
    x = mxfp4.dequantize(packed, scales).astype(np.float32)
    c2, s2 = mxfp4.quantize(x)
    np.testing.assert_array_equal(s2, scales)
    np.testing.assert_array_equal(c2, packed)                     # dequant(quant(x)) = x, sign of zero included
    y = (rng.standard_normal((rows, G * 32)) * 3).astype(np.float32)
    c, s = mxfp4.quantize(y)
    c3, s3 = mxfp4.quantize(mxfp4.dequantize(c, s).astype(np.float32))
    # quant . dequant . quant = quant, except that a group whose maximum was rounded down
    # below 4*s may pick a smaller scale; its values must still be reproduced exactly
    np.testing.assert_array_equal(mxfp4.dequantize(c3, s3), mxfp4.dequantize(c, s))


def test_error_bound():
    """|dequant - y| <= half the local E2M1 step times s; < 2 s when saturating; 4 <= amax/s < 8."""
    rng = np.random.default_rng(11)
    y = (rng.standard_normal((64, 256)) * np.exp(rng.uniform(-5, 5, size=(64, 1)))).astype(np.float32)
    y[::7, ::13] *= 40
    c, s = mxfp4.quantize(y)
    d = mxfp4.dequantize(c, s)
    sc = np.repeat(np.ldexp(1.0, s.astype(np.int64) - 127), 32, axis=1)
    v = np.abs(y.astype(np.float64)) / sc
    err = np.abs(d - y.astype(np.float64)) / sc
    assert np.all(err[v <= 2] <= 0.25)
    assert np.all(err[(v > 2) & (v <= 4)] <= 0.5)
    assert np.all(err[(v > 4) & (v <= 6)] <= 1.0)
    assert np.all(err[v > 6] < 2.0)
    ratio = np.max(v.reshape(64, -1, 32), axis=-1)
    assert np.all((ratio >= 4) & (ratio < 8))


def test_group_independence():
    rng = np.random.default_rng(3)
    y = rng.standard_normal((4, 128)).astype(np.float32)
    c0, s0 = mxfp4.quantize(y)
    y2 = y.copy()
    y2[:, 32:64] *= 1000.0
    c1, s1 = mxfp4.quantize(y2)
    keep = np.r_[0:16, 32:64]
    np.testing.assert_array_equal(c0[:, keep], c1[:, keep])
    np.testing.assert_array_equal(s0[:, [0, 2, 3]], s1[:, [0, 2, 3]])
    assert np.any(s0[:, 1] != s1[:, 1])
