"""CPU oracle of the 8-bit expert-weight format (Section 6 calls weight quantisation
orthogonal to budget allocation; this is the variant for the weight-bound regimes).

TEST INFRASTRUCTURE, NOT THE PRODUCT (see oracle/__init__.py).

Format (the OCP 8-bit floating point specification's E4M3): a byte is sign (1 bit),
exponent e (4 bits, bias 7), mantissa m (3 bits):
    e > 0 : (-1)^s * 2^(e-7) * (1 + m/8)
    e = 0 : (-1)^s * 2^(-6) * (m/8)             (subnormals; m = 0 is zero)
    e = 15, m = 7 : NaN (never produced here); there are no infinities; the largest
    finite magnitude is 2^8 * 1.75 = 448.
A weight matrix W[k][n] is stored per output column n as codes q[k][n] and one fp32
scale:
    scale[n] = max_k |W[k][n]| / 448     (fp32 division; 1 if the column is all zero)
    q[k][n]  = E4M3 code nearest to W[k][n] / scale[n]   (fp32 division; ties to the
               code with even mantissa; magnitudes above 448 saturate to 448)
and stands for the value  decode(q[k][n]) * scale[n].

Everything that decides a code is done in fp32, as the device does it.
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0


def e4m3_decode_byte(code: int) -> float:
    """The definition, one byte."""
    s = -1.0 if code & 0x80 else 1.0
    e, m = (code >> 3) & 0xF, code & 0x7
    if e == 15 and m == 7:
        return float("nan")
    if e == 0:
        return s * (m / 8.0) * 2.0 ** -6
    return s * (1.0 + m / 8.0) * 2.0 ** (e - 7)


_POS = np.array([e4m3_decode_byte(c) for c in range(0x7F)], dtype=np.float64)   # codes 0x00..0x7E


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    codes = np.asarray(codes, dtype=np.uint8)
    table = np.array([e4m3_decode_byte(c) for c in range(256)], dtype=np.float64)
    return table[codes]


def e4m3_encode(y: np.ndarray) -> np.ndarray:
    """Nearest code, ties to the even mantissa, saturating; y is taken as fp32."""
    y = np.asarray(y, dtype=np.float32).astype(np.float64)
    a = np.minimum(np.abs(y), E4M3_MAX)
    hi = np.searchsorted(_POS, a, side="left")            # first table value >= a
    hi = np.minimum(hi, len(_POS) - 1)
    lo = np.maximum(hi - 1, 0)
    d_lo, d_hi = a - _POS[lo], _POS[hi] - a
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    return np.where(np.signbit(y), code | 0x80, code).astype(np.uint8)


def quantise_columns(W: np.ndarray):
    """W [..., Kd, N] (values exactly representable in fp32) -> (codes uint8 [..., Kd, N],
    scale fp32 [..., N])."""
    W32 = np.asarray(W, dtype=np.float32)
    amax = np.max(np.abs(W32), axis=-2)
    scale = np.where(amax > 0, amax / np.float32(E4M3_MAX), np.float32(1.0)).astype(np.float32)
    y = (W32 / scale[..., None, :]).astype(np.float32)
    return e4m3_encode(y), scale


def dequantise(codes: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """The values the stored matrix stands for, fp64."""
    return e4m3_decode(codes) * np.asarray(scale, dtype=np.float64)[..., None, :]
