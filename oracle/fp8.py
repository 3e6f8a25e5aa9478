"""The 8-bit floating-point format E4M3 of the OCP 8-bit Floating Point Specification
(OFP8), decoded from its definition.

TEST INFRASTRUCTURE ONLY, like the rest of this package.

A code is 1 sign bit, 4 exponent bits (bias 7) and 3 mantissa bits:
    exponent field 0      subnormal:  (-1)^s * 2^-6 * (m / 8)
    exponent field 1..15  normal:     (-1)^s * 2^(e - 7) * (1 + m / 8)
except that exponent 15 with mantissa 7 is NaN; the format has no infinities, so its
largest magnitude is 2^8 * 1.75 = 448.
"""
from __future__ import annotations

import numpy as np


def e4m3_value(code: int) -> float:
    code = int(code)
    if not 0 <= code <= 255:
        raise ValueError("an E4M3 code is one byte")
    sign = -1.0 if code & 0x80 else 1.0
    e = (code >> 3) & 0xF
    m = code & 0x7
    if e == 15 and m == 7:
        return float("nan")
    if e == 0:
        return sign * (m / 8.0) * 2.0 ** -6
    return sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)


E4M3_TABLE = np.array([e4m3_value(c) for c in range(256)], dtype=np.float64)


def decode_e4m3(codes) -> np.ndarray:
    """uint8 codes -> float32 values of the same shape (every E4M3 value is a float32)."""
    codes = np.asarray(codes)
    if codes.dtype != np.uint8:
        raise TypeError("E4M3 codes travel as uint8")
    return E4M3_TABLE.astype(np.float32)[codes]
