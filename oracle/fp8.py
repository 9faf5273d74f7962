"""CPU oracle: the 8-bit floating-point format of the fp8 KV-cache variant.  TEST INFRASTRUCTURE ONLY.

E4M3 as the OCP 8-bit floating point specification defines it ("E4M3", the finite-only variant
also written e4m3fn): 1 sign bit, 4 exponent bits with bias 7, 3 mantissa bits; exponent field 0
holds subnormals (mantissa * 2^-9); there are no infinities; only S.1111.111 is NaN; the largest
finite value is S.1111.110 = 448.

Encoding rounds to the nearest representable value, ties to the even mantissa, and saturates:
anything that would round beyond 448 becomes +-448; NaN stays NaN.
"""
from __future__ import annotations

import numpy as np

MAX = 448.0


def decode_one(code: int) -> float:
    sign = -1.0 if code & 0x80 else 1.0
    e = (code >> 3) & 0xF
    m = code & 7
    if e == 15 and m == 7:
        return float("nan")
    if e == 0:
        return sign * m * 2.0 ** -9
    return sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)


TABLE = np.array([decode_one(c) for c in range(256)], np.float64)


def decode(codes) -> np.ndarray:
    return TABLE[np.asarray(codes, np.uint8)]


def encode_one(x: float) -> int:
    if x != x:
        return 0x7F
    sign = 0x80 if (x < 0 or (x == 0 and np.signbit(x))) else 0
    a = abs(float(x))
    if a >= MAX:
        return sign | 0x7E
    # spacing of the grid around a: 2^-9 below the smallest normal, 2^(e-3) in binade e
    e = max(int(np.floor(np.log2(a))) if a > 0 else -7, -6)
    step = 2.0 ** (e - 3)
    q = a / step                       # exact: a power-of-two scaling
    n = int(np.floor(q))
    frac = q - n
    if frac > 0.5 or (frac == 0.5 and n % 2 == 1):
        n += 1
    val = n * step
    if val > MAX:
        val = MAX
    # find the code of val (it is on the grid by construction)
    if val < 2.0 ** -6:
        return sign | int(round(val * 2.0 ** 9))
    ee = int(np.floor(np.log2(val)))
    mant = int(round((val / 2.0 ** ee - 1.0) * 8))
    return sign | ((ee + 7) << 3) | mant


def encode(x) -> np.ndarray:
    """encode_one over an array: the nearest of the 127 non-negative grid values (their codes are
    their ranks), ties to the even code, the sign bit on top.  Same results as encode_one (pinned)."""
    x = np.asarray(x, np.float64)
    grid = TABLE[:0x7F]                                  # codes 0x00 .. 0x7E: ascending, 0 .. 448
    a = np.minimum(np.abs(x), MAX)
    a = np.where(np.isnan(a), 0.0, a)
    hi = np.clip(np.searchsorted(grid, a, side="left"), 1, 0x7E)
    lo = hi - 1
    d_lo, d_hi = a - grid[lo], grid[hi] - a
    code = np.where(d_lo < d_hi, lo, np.where(d_hi < d_lo, hi, np.where(lo % 2 == 0, lo, hi)))
    code = np.where(a == grid[hi], hi, code)
    out = (code | np.where(np.signbit(x), 0x80, 0)).astype(np.uint8)
    return np.where(np.isnan(x), np.uint8(0x7F), out).astype(np.uint8)
