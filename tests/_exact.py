"""Exact-arithmetic helpers used to pin the oracle (independent of oracle/).

Everything here works on Python ints / Fractions so that no floating-point
rounding of the host can hide a mistake in the code under test.
"""
from __future__ import annotations

import struct
from fractions import Fraction

E2M1_VALUES = [Fraction(0), Fraction(1, 2), Fraction(1), Fraction(3, 2),
               Fraction(2), Fraction(3), Fraction(4), Fraction(6)]


def f32_bits(x: float) -> int:
    return struct.unpack("<I", struct.pack("<f", x))[0]


def bits_f32(u: int) -> float:
    return struct.unpack("<f", struct.pack("<I", u & 0xFFFFFFFF))[0]


def to_f32(x) -> float:
    """Round a Python float/Fraction to the nearest binary32 (ties to even)."""
    return struct.unpack("<f", struct.pack("<f", float(x)))[0]


def e4m3_value(b: int) -> Fraction:
    """Value of an E4M3 byte by the format's definition (bias 7, subnormals)."""
    e, m = (b >> 3) & 15, b & 7
    assert not (e == 15 and m == 7)
    mag = Fraction(m, 8) * Fraction(1, 64) if e == 0 else (1 + Fraction(m, 8)) * Fraction(2) ** (e - 7)
    return -mag if b & 0x80 else mag


E4M3_POS = [e4m3_value(b) for b in range(0x7F)]     # 0x00 .. 0x7E, increasing


def nearest_even(x: Fraction, values) -> int:
    """Index of the value nearest to x (values increasing); ties go to the even
    index; x above the last value saturates to it."""
    if x >= values[-1]:
        return len(values) - 1
    best, best_d = 0, None
    for k, v in enumerate(values):
        d = abs(x - v)
        if best_d is None or d < best_d or (d == best_d and k % 2 == 0 and best % 2 == 1):
            best, best_d = k, d
    return best


def e2m1_nearest(y: Fraction) -> int:
    """E2M1 code (sign<<3 | index) of exact y by nearest value, ties to even index."""
    k = nearest_even(abs(y), E2M1_VALUES)
    return (8 if y < 0 else 0) | k


def philox4x32_10(ctr, key):
    """Big-integer Philox4x32-10 written from the SC'11 definition."""
    M0, M1 = 0xD2511F53, 0xCD9E8D57
    W0, W1 = 0x9E3779B9, 0xBB67AE85
    c = list(ctr)
    k = list(key)
    mask = (1 << 32) - 1
    for _ in range(10):
        p0 = M0 * c[0]
        p1 = M1 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & mask, p1 & mask,
             ((p0 >> 32) ^ c[3] ^ k[1]) & mask, p0 & mask]
        k = [(k[0] + W0) & mask, (k[1] + W1) & mask]
    return tuple(c)
