"""The 8-bit (E4M3, per-column scale) expert-weight format: oracle pins (CPU).

The decode table is checked against values written out from the format's definition,
the encoder against the exact nearest / ties-to-even rule evaluated with rationals over
all codes (brute force), and the column quantiser against the properties its definition
implies.
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle import quant


def exact(code):   # the definition again, in rationals
    s = -1 if code & 0x80 else 1
    e, m = (code >> 3) & 0xF, code & 7
    if e == 0:
        return s * Fraction(m, 8) * Fraction(1, 64)
    return s * (1 + Fraction(m, 8)) * (Fraction(2) ** (e - 7))


def test_decode_known_values():
    known = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x0F: 1.875 * 2.0 ** -6,
             0x30: 0.5, 0x38: 1.0, 0x39: 1.125, 0x3F: 1.875, 0x40: 2.0, 0x78: 256.0, 0x7E: 448.0,
             0x80: -0.0, 0xB8: -1.0, 0xFE: -448.0}
    for code, value in known.items():
        assert quant.e4m3_decode_byte(code) == value
    assert np.isnan(quant.e4m3_decode_byte(0x7F)) and np.isnan(quant.e4m3_decode_byte(0xFF))
    table = quant.e4m3_decode(np.arange(256, dtype=np.uint8))
    pos = table[:0x7F]
    assert np.all(np.diff(pos) > 0) and len(pos) == 127          # 127 finite values, increasing
    assert np.array_equal(table[0x80:0xFF], -pos)
    for c in range(0x7F):
        assert Fraction(float(table[c])) == exact(c)


def test_encode_round_trip_and_ties():
    codes = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], dtype=np.uint8)
    assert np.array_equal(quant.e4m3_encode(quant.e4m3_decode(codes)), codes)
    cases = {1.0625: 0x38, 1.1875: 0x3A, 0.9688: 0x38,       # midpoints go to the even mantissa
             2.0 ** -10: 0x00, 3 * 2.0 ** -10: 0x02,         # subnormal midpoints
             15 * 2.0 ** -10: 0x08,                          # largest subnormal / smallest normal midpoint
             448.0: 0x7E, 449.0: 0x7E, 464.0: 0x7E, 1e9: 0x7E, -1e9: 0xFE,
             432.0: 0x7E, 431.9: 0x7D, 0.0: 0x00}
    cases[0.96875] = cases.pop(0.9688)     # exactly half way between 0.9375 (0x37) and 1.0 (0x38)
    for value, code in cases.items():
        assert int(quant.e4m3_encode(np.float32(value))) == code, (value, code)


def test_encode_is_nearest_with_even_ties_brute_force():
    rng = np.random.default_rng(5)
    finite = [c for c in range(0x7F)]
    ys = np.concatenate([rng.normal(0, 100, 400), rng.normal(0, 1, 400), rng.normal(0, 0.01, 400),
                         np.array([(float(exact(c)) + float(exact(c + 1))) / 2 for c in range(0x7E)])])
    ys = ys.astype(np.float32)
    got = quant.e4m3_encode(ys)
    for y, g in zip(ys, got):
        a = min(abs(Fraction(float(y))), Fraction(448))
        best = min(finite, key=lambda c: (abs(exact(c) - a), c & 1))
        assert (int(g) & 0x7F) == best, (float(y), int(g), best)
        assert bool(int(g) & 0x80) == bool(np.signbit(y))


def test_quantise_columns_properties():
    rng = np.random.default_rng(6)
    W = rng.normal(0, 0.02, (3, 96, 40)).astype(np.float32)
    W[1, :, 7] = 0.0                                     # an all-zero column
    codes, scale = quant.quantise_columns(W)
    assert codes.shape == W.shape and scale.shape == (3, 40) and scale.dtype == np.float32
    amax = np.abs(W).max(axis=-2)
    assert np.array_equal(scale[amax > 0], (amax / np.float32(448.0))[amax > 0])
    assert scale[1, 7] == 1.0 and not codes[1, :, 7].any()
    # the largest entry of a column lands on +-448
    top = np.abs(quant.e4m3_decode(codes)).max(axis=-2)
    assert np.all(top[amax > 0] == 448.0)
    # error bound: half a mantissa step (2^-4 relative) or half a subnormal step
    back = quant.dequantise(codes, scale)
    bound = np.maximum(np.abs(W) * 2.0 ** -4, scale[:, None, :] * 2.0 ** -10) * (1 + 1e-6)
    assert np.all(np.abs(back - W) <= bound)
    # signs survive, zeros stay zeros
    assert np.array_equal(np.signbit(back[W != 0]), np.signbit(W[W != 0]))
