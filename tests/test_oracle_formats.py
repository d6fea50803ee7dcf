"""Pins for the oracle's number formats: E2M1, E4M3, BF16.

Each check compares the oracle with something that is not the oracle: values
the paper prints (tests/golden/format_facts.txt), the formats' definitions
evaluated in exact rational arithmetic, or torch's own casts.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import ref
from tests._exact import (E2M1_VALUES, E4M3_POS, bits_f32, e2m1_nearest, e4m3_value, f32_bits,
                          nearest_even, to_f32)


def _facts(golden_dir):
    out = []
    for line in (golden_dir / "format_facts.txt").read_text().splitlines():
        line = line.strip()
        if line and not line.startswith("#"):
            out.append(line.split())
    return out


def test_e2m1_grid_matches_paper(golden_dir):
    (grid,) = [f[1] for f in _facts(golden_dir) if f[0] == "e2m1_grid"]
    want = [float(v) for v in grid.split(",")]
    assert [ref.e2m1_decode(k) for k in range(8)] == want
    assert [ref.e2m1_decode(8 | k) for k in range(8)] == [-v for v in want]
    # -0 keeps its sign
    assert np.signbit(np.float32(ref.e2m1_decode(8)))
    # the 16 codes give 15 distinct values plus a signed zero
    assert len({ref.e2m1_decode(c) for c in range(16)}) == 15


def test_e2m1_paper_roundings(golden_dir):
    for f in _facts(golden_dir):
        if f[0] == "e2m1_round":
            y, want = float(f[1]), float(f[2])
            assert ref.e2m1_decode(ref.e2m1_rtn(to_f32(y))) == want, f
            assert ref.e2m1_decode(ref.e2m1_rtn(to_f32(-y))) == -want, f


def test_e2m1_step_sizes(golden_dir):
    vals = sorted({abs(ref.e2m1_decode(c)) for c in range(16)})
    for f in _facts(golden_dir):
        if f[0] == "e2m1_step":
            lo, hi, step = float(f[1]), float(f[2]), float(f[3])
            seg = [v for v in vals if lo <= v <= hi]
            assert all(b - a == step for a, b in zip(seg, seg[1:])), f


def test_e2m1_rtn_is_nearest_with_ties_to_even_exact():
    """Eq. (3) as coded == nearest grid value in exact arithmetic, half-even."""
    rng = np.random.default_rng(1)
    samples = list(rng.uniform(-7.5, 7.5, 4000).astype(np.float32))
    samples += list((rng.standard_normal(2000) * 1e-3).astype(np.float32))
    # every midpoint and grid point, and their fp32 neighbours
    for v in [0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 0.5, 1, 1.5, 2, 3, 4, 6, 7, 100.0]:
        u = f32_bits(v)
        for d in (-2, -1, 0, 1, 2):
            samples += [bits_f32(u + d), -bits_f32(u + d)]
    samples += [0.0, -0.0, 1e-45, -1e-45, 1e-38, 3.0e38, -3.0e38]
    for y in samples:
        y = float(np.float32(y))
        got = ref.e2m1_rtn(y)
        want = e2m1_nearest(Fraction(y))
        if y == 0.0:
            want = 8 if np.signbit(np.float32(y)) else 0
        assert got == want, (y, got, want)


def test_e2m1_rtn_tie_table():
    ties = {0.25: 0.0, 0.75: 1.0, 1.25: 1.0, 1.75: 2.0, 2.5: 2.0, 3.5: 4.0, 5.0: 4.0}
    for y, want in ties.items():
        assert ref.e2m1_decode(ref.e2m1_rtn(y)) == want
        assert ref.e2m1_decode(ref.e2m1_rtn(-y)) == -want
    # sign of a value that rounds to zero is kept
    assert ref.e2m1_rtn(-0.1) == 8 and ref.e2m1_rtn(0.1) == 0


def test_e2m1_rtn_monotone_and_idempotent():
    ys = np.linspace(-8, 8, 6401, dtype=np.float32)
    vals = [ref.e2m1_decode(ref.e2m1_rtn(float(y))) for y in ys]
    assert all(b >= a for a, b in zip(vals, vals[1:]))
    for c in range(16):
        assert ref.e2m1_rtn(ref.e2m1_decode(c)) == c


def test_e2m1_sr_bounds_and_probability():
    rng = np.random.default_rng(2)
    for y in rng.uniform(-7, 7, 500).astype(np.float32):
        y = float(y)
        a = min(abs(y), 6.0)
        lo = max(v for v in E2M1_VALUES if v <= Fraction(a))
        his = [v for v in E2M1_VALUES if v > Fraction(a)]
        hi = min(his) if his else lo
        p = Fraction(0) if hi == lo else (Fraction(a) - lo) / (hi - lo)
        for u in (0.0, 0.25, 0.5, 0.75, 1 - 2.0 ** -24):
            code = ref.e2m1_sr(y, u)
            mag = Fraction(abs(ref.e2m1_decode(code)))
            assert mag in (lo, hi)
            assert (mag == hi and hi != lo) == (Fraction(u) < p and hi != lo), (y, u)
            assert bool(code & 8) == (y < 0)
    # u == p exactly does not round up (the rule is u < p): 1.25 has p = 1/2,
    # 2.25 has p = 1/4, 5.5 has p = 3/4
    for y, u, dn, up in ((1.25, 0.5, 1.0, 1.5), (2.25, 0.25, 2.0, 3.0), (5.5, 0.75, 4.0, 6.0)):
        assert ref.e2m1_decode(ref.e2m1_sr(y, u)) == dn
        assert ref.e2m1_decode(ref.e2m1_sr(y, u - 2.0 ** -24)) == up
        assert ref.e2m1_decode(ref.e2m1_sr(-y, u)) == -dn
    # magnitudes above 6 saturate
    assert ref.e2m1_sr(7.5, 0.0) == 7 and ref.e2m1_sr(-1e9, 0.5) == 15
    # a value on the grid never moves, whatever u is
    for c in range(16):
        for u in (0.0, 0.999):
            assert ref.e2m1_sr(ref.e2m1_decode(c), u) == c


def test_e4m3_decode_all_bytes_by_definition():
    for b in range(256):
        if (b & 0x7F) == 0x7F:
            assert np.isnan(ref.e4m3_decode(b))
            continue
        assert Fraction(ref.e4m3_decode(b)) == e4m3_value(b)
    assert ref.e4m3_decode(0x7E) == 448.0
    assert ref.e4m3_decode(0x01) == 2.0 ** -9
    assert ref.e4m3_decode(0x08) == 2.0 ** -6


def test_e4m3_paper_facts(golden_dir):
    for f in _facts(golden_dir):
        if f[0] == "e4m3_round":
            assert ref.e4m3_decode(ref.e4m3_encode(to_f32(float(f[1])))) == float(f[2]), f
        elif f[0] == "e4m3_max":
            assert max(ref.e4m3_decode(b) for b in range(0x7F)) == float(f[1])
        elif f[0] == "e4m3_exact":
            assert ref.e4m3_decode(ref.e4m3_encode(float(f[1]))) == float(f[1]), f
        elif f[0] == "e4m3_overflow":
            # saturates to the maximum instead of producing the NaN pattern
            assert ref.e4m3_encode(float(f[1])) == 0x7E, f


def test_e4m3_encode_roundtrip_monotone_saturating():
    for b in range(0x7F):
        assert ref.e4m3_encode(ref.e4m3_decode(b)) == b
    xs = np.concatenate([np.linspace(0, 500, 20001), np.geomspace(1e-6, 500, 5000)]).astype(np.float32)
    xs.sort()
    enc = [ref.e4m3_encode(float(x)) for x in xs]
    assert all(b >= a for a, b in zip(enc, enc[1:]))
    for x in (448.0, 449.0, 463.9, 464.0, 480.0, 1e9, float(np.float32(3e38)), float("inf")):
        assert ref.e4m3_encode(x) == 0x7E
    assert ref.e4m3_encode(0.0) == 0 and ref.e4m3_encode(-0.0) == 0


def test_e4m3_encode_is_nearest_of_127_exact():
    rng = np.random.default_rng(3)
    xs = list(rng.uniform(0, 460, 1500).astype(np.float32))
    xs += list(np.exp2(rng.uniform(-14, 9, 1500)).astype(np.float32))
    # all midpoints between neighbours and their fp32 neighbours
    for a, b in zip(E4M3_POS, E4M3_POS[1:]):
        mid = float((a + b) / 2)
        u = f32_bits(mid)
        xs += [bits_f32(u - 1), mid, bits_f32(u + 1)]
    for x in xs:
        x = float(np.float32(x))
        want = nearest_even(Fraction(x), E4M3_POS)
        assert ref.e4m3_encode(x) == want, (x, ref.e4m3_encode(x), want)


def test_e4m3_encode_matches_torch_in_range():
    rng = np.random.default_rng(4)
    xs = np.concatenate([rng.uniform(0, 447.9, 20000), np.exp2(rng.uniform(-12, 8.8, 20000))])
    xs = xs.astype(np.float32)
    t = torch.from_numpy(xs).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([ref.e4m3_encode(float(x)) for x in xs], dtype=np.uint8)
    assert np.array_equal(got, t)
    # the range helper agrees with the scalar entry point
    first = f32_bits(1.0)
    rng_out = ref.e4m3_encode_bits_range(first, 4096)
    assert all(rng_out[i] == ref.e4m3_encode(bits_f32(first + i)) for i in range(0, 4096, 97))


def test_bf16_conversions_match_torch():
    rng = np.random.default_rng(5)
    xs = np.concatenate([rng.standard_normal(20000) * np.exp2(rng.integers(-30, 30, 20000)),
                         [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895e38, 3.4e38]]).astype(np.float32)
    want = torch.from_numpy(xs).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([ref.f32_to_bf16(float(x)) for x in xs], dtype=np.uint16)
    assert np.array_equal(got, want)
    # ties to even on the exact halfway patterns
    assert ref.f32_to_bf16(bits_f32(0x3F808000)) == 0x3F80
    assert ref.f32_to_bf16(bits_f32(0x3F818000)) == 0x3F82
    for h in list(range(0, 0x7F80, 257)) + [0x8000, 0x0001, 0x7F7F, 0xFF7F]:
        assert f32_bits(ref.bf16_to_f32(h)) == h << 16


@pytest.mark.parametrize("first", [0x00000000, 0x3E000000, 0x40000000, 0x40BFFF00, 0xC0000000])
def test_e2m1_range_helper_agrees_with_scalar(first):
    out = ref.e2m1_rtn_bits_range(first, 1 << 12)
    for i in range(0, 1 << 12, 61):
        assert out[i] == ref.e2m1_rtn(bits_f32(first + i))
