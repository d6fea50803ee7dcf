"""CPU: what the reciprocal reading of Eq. (3) changes.

Eq. (3) rounds X / (alpha * Delta).  The oracle (and the kernels) multiply by the rounded
reciprocal instead, y = fl(v * fl(1 / dec)), one division per block and candidate rather than
one per element.  This test counts, on an activation-like tensor whose tensor scale has a short
mantissa (max|x| = 1000 gives alpha = 1000/1536), where that matters: the codes of
  (a) y = fl(v * fl(1/dec))      -- the reading,
  (b) y = fl(v / dec)            -- a correctly rounded fp32 division per element,
  (c) the exact rational quotient v / dec,
each rounded to the E2M1 grid with ties to even.  (a) and (b) are two fp32 renderings of (c);
they can differ from each other only where the quotient lies within an ulp of a rounding
midpoint.  On this tensor they differ on about one code in ten thousand (101 of 1,048,576), and
on every one of those the exact quotient rounds as the reading does: the division's result
lands exactly on the midpoint and takes the tie rule, while the true quotient lies just beside it.
"""
from fractions import Fraction

import numpy as np
import torch

from oracle import ref
from paper_2512_02010_amd import workloads as wl
from tests._exact import e2m1_nearest, e4m3_value

MIDPOINTS = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0], np.float32)
GRID = np.array([0, .5, 1, 1.5, 2, 3, 4, 6], np.float32)


def _codes(y: np.ndarray) -> np.ndarray:
    """E2M1 index of |y| (fp32), nearest value, ties to the even index, saturating."""
    a = np.minimum(np.abs(y), np.float32(6.0))
    k = np.zeros(a.shape, np.int64)
    for i, m in enumerate(MIDPOINTS):
        k += (a > m) | ((a == m) & (i % 2 == 1))      # at a midpoint go up only towards an even index
    return k


def test_reciprocal_multiply_against_division_and_exact_quotient():
    x = wl.make("c3", 1024, 1024)
    x[0, 0] = 1000.0                                   # the short-mantissa tensor scale
    xb = wl.bf16_bits(x)
    alpha = ref.tensor_scale(xb)
    assert np.float32(alpha) == np.float32(1000.0) / np.float32(1536.0)
    _, scales, _ = ref.quantize(xb, alpha)
    dec = np.array([ref.e4m3_decode(int(s)) for s in range(127)], np.float32)[scales] * np.float32(alpha)
    v = x.float().numpy().reshape(1024, 64, 16)
    dec3 = dec[:, :, None]
    with np.errstate(divide="ignore", invalid="ignore"):
        enc = np.where(dec3 == 0, np.float32(0), np.float32(1.0) / dec3).astype(np.float32)
        y_rec = (v * enc).astype(np.float32)
        y_div = np.where(dec3 == 0, np.float32(0), v / dec3).astype(np.float32)
    ka, kb = _codes(y_rec), _codes(y_div)
    diff = np.argwhere(ka != kb)
    n = v.size
    # rare: a few elements per million
    assert 0 < len(diff) < n * 5e-4, len(diff)
    agree_a = agree_b = 0
    for r, b, i in diff:
        q = Fraction(float(v[r, b, i])) / Fraction(float(dec[r, b]))
        kc = e2m1_nearest(q) & 7
        assert kc in (ka[r, b, i], kb[r, b, i])
        agree_a += kc == ka[r, b, i]
        agree_b += kc == kb[r, b, i]
        # only within an ulp or two of a rounding midpoint can the two renderings part
        m = MIDPOINTS[np.argmin(np.abs(MIDPOINTS - abs(float(q))))]
        assert abs(abs(q) - Fraction(float(m))) <= Fraction(float(m)) * Fraction(3, 2 ** 24)
    assert agree_a + agree_b == len(diff)
    # where they part, the division has rounded onto the midpoint itself; the exact quotient
    # lies beside it, on the side the reading took
    assert agree_a >= agree_b
    print(f"\nEq. (3) reading: {len(diff)} of {n} codes differ between reciprocal-multiply and per-element "
          f"division; the exact quotient sides with the reading on {agree_a}, with the division on {agree_b}")
