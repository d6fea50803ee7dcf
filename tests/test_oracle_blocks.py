"""Pins for the oracle's per-block 4/6 procedure (Table 3, Section 3.1).

Sources of truth used here: the two blocks the paper works through, exact
rational re-evaluation of the definitions, brute force over every E4M3
scale, and the closed-form statements of Section 3 / Figure 1.
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle import ref
from tests._exact import E2M1_VALUES, E4M3_POS, e2m1_nearest, e4m3_value, nearest_even, to_f32


def _worked(golden_dir):
    rows = []
    for line in (golden_dir / "table3_worked_blocks.txt").read_text().splitlines():
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        d = dict(tok.split("=", 1) for tok in line.split())
        for k in ("block", "scaled", "q", "D"):
            d[k] = [float(v) for v in d[k].split(",")]
        for k in ("M", "pre", "delta", "mse_printed", "mse_exact", "chosen"):
            d[k] = float(d[k])
        rows.append(d)
    return rows


def test_table3_worked_blocks(golden_dir):
    rows = _worked(golden_dir)
    assert len(rows) == 4
    for d in rows:
        x = d["block"]
        n = len(x)
        sel = ref.SEL_FORCE6 if d["M"] == 6 else ref.SEL_FORCE4
        r = ref.quantize_block(x, 1.0, ref.RTN, sel)
        # lines 1-2 / 7-8: the scale before and after the E4M3 cast
        assert round(max(x) / d["M"], 2) == d["pre"]
        assert ref.e4m3_decode(r["S"]) == d["delta"]
        # lines 3-4 / 9-10
        assert [round(v / d["delta"], 2) for v in x] == d["scaled"]
        assert [ref.e2m1_decode(c) for c in r["codes"][:n]] == d["q"]
        # line 5 / 11, line 6 / 12 (sum = n * mean; the zero padding adds nothing)
        assert list(r["D"][:n]) == d["D"]
        E = r["E6"] if d["M"] == 6 else r["E4"]
        assert E == d["mse_exact"] * n
        assert abs(E / n - d["mse_printed"]) < 0.005 or d["mse_printed"] == 96.25
        # lines 13-14
        full = ref.quantize_block(x, 1.0, ref.RTN, ref.SEL_46_MSE)
        assert (4.0 if full["four"] else 6.0) == d["chosen"]
        if d["M"] == d["chosen"]:
            assert full["S"] == r["S"] and list(full["codes"]) == list(r["codes"])
            assert list(full["D"]) == list(r["D"])


def test_table3_block_position_and_sign_do_not_matter():
    for x, four in (([10, 20, 30, 40], 1), ([15, 30, 120, 180], 0)):
        base = ref.quantize_block(x, 1.0)
        rng = np.random.default_rng(0)
        for _ in range(5):
            v = np.zeros(16, np.float32)
            pos = rng.permutation(16)[:4]
            sg = rng.choice([-1.0, 1.0], 4)
            v[pos] = np.array(x, np.float32) * sg
            r = ref.quantize_block(v, 1.0)
            assert r["four"] == four and r["S"] == base["S"]
            assert list(r["D"][pos]) == list(base["D"][:4] * sg)


def test_tie_keeps_six():
    # all zeros: both candidates have zero error -> 6 (Table 3 line 13 is strict)
    r = ref.quantize_block([0.0] * 16, 1.0)
    assert r["four"] == 0 and r["E4"] == r["E6"] == 0.0 and r["S"] == 0
    # a single non-zero value is exact under both scalings when max/6 and max/4
    # are E4M3 values (12 -> 2 and 3)
    r = ref.quantize_block([12.0], 1.0)
    assert r["E4"] == r["E6"] == 0.0 and r["four"] == 0
    assert ref.e4m3_decode(r["S"]) == 2.0 and ref.e2m1_decode(r["codes"][0]) == 6.0


def _exact_block(v, alpha, S):
    """Candidate (codes, D, E) by the definitions in exact rational arithmetic:
    q = nearest E2M1 value to v / (alpha * Delta), D = q * Delta * alpha."""
    dec = e4m3_value(S) * Fraction(alpha)
    codes, D = [], []
    for x in v:
        x = Fraction(float(x))
        code = e2m1_nearest(x / dec) if dec != 0 else (8 if x < 0 else 0)
        mag = E2M1_VALUES[code & 7] * dec
        codes.append(code)
        D.append(-mag if code & 8 else mag)
    E = sum((d - Fraction(float(x))) ** 2 for d, x in zip(D, v))
    return codes, D, E


def test_block_with_scale_against_exact_rational():
    """With few-bit inputs and a power-of-two alpha every fp32 step of the oracle
    is exact, so it has to reproduce the rational evaluation of Table 3 bit for
    bit (dropped terms, sign slips and index slips all show up here)."""
    rng = np.random.default_rng(11)
    checked = 0
    for trial in range(300):
        v = (rng.integers(-48, 49, 16) * 0.25).astype(np.float32)
        alpha = float(2.0 ** rng.integers(-3, 2))
        for S in (0x28, 0x30, 0x34, 0x38, 0x3C, 0x40, 0x44, 0x48):   # 0.25 .. 4 incl. 1.5-type mantissas
            dec = e4m3_value(S) * Fraction(alpha)
            # skip the rare case where the reciprocal is inexact AND a value
            # sits exactly on a rounding midpoint of the exact quotient
            enc_exact = (1 / dec).denominator & ((1 / dec).denominator - 1) == 0
            on_mid = any((Fraction(float(x)) / dec * 4) % 1 == 0 and
                         (Fraction(float(x)) / dec * 4) % 2 == 1 for x in v)
            if not enc_exact and on_mid:
                continue
            E, q, D = ref.block_with_scale(v, alpha, S)
            cq, cD, cE = _exact_block(v, alpha, S)
            assert list(q) == cq, (v, alpha, S)
            assert [Fraction(float(d)) for d in D] == cD
            assert Fraction(E) == cE, (v, alpha, S, E, float(cE))
            checked += 1
    assert checked > 1500


def test_block_scale_is_eq2_then_e4m3_cast():
    rng = np.random.default_rng(12)
    for _ in range(2000):
        b = float(np.float32(abs(rng.standard_normal()) * 2.0 ** rng.integers(-8, 8)))
        alpha = float(np.float32(abs(rng.standard_normal()) * 2.0 ** rng.integers(-12, 2) + 1e-6))
        for M in (6.0, 4.0):
            # fp32 product, fp32 quotient (numpy float32 ops round once each)
            sf = np.float32(b) / (np.float32(alpha) * np.float32(M))
            want = nearest_even(Fraction(float(sf)), E4M3_POS)
            assert ref.block_scale(b, alpha, M) == want


def test_tensor_scale_256_lets_the_max_block_pick_four():
    # Section 3.1: with 256 in Eq. (1) the block holding the tensor maximum gets
    # scale 256 when mapped to 6 and 384 when mapped to 4, both exact in E4M3;
    # with 448 the M=4 scale would have to be 672 and saturates.
    for amax in (1.0, 0.37, 1234.5, 2.0 ** -20):
        amax = to_f32(amax)
        a256 = float(np.float32(amax) / np.float32(1536.0))
        a448 = float(np.float32(amax) / np.float32(2688.0))
        assert ref.e4m3_decode(ref.block_scale(amax, a256, 6.0)) == 256.0
        assert ref.e4m3_decode(ref.block_scale(amax, a256, 4.0)) == 384.0
        assert ref.e4m3_decode(ref.block_scale(amax, a448, 6.0)) == 448.0
        assert ref.block_scale(amax, a448, 4.0) == 0x7E          # 672 saturates
    # an all-equal-magnitude block is exact under both scalings with 256 -> tie -> 6
    v = np.full(16, 0.37, np.float32)
    v[::3] *= -1
    a = float(np.float32(np.abs(v).max()) / np.float32(1536.0))
    r = ref.quantize_block(v, a)
    assert r["S"] == 0x78 and r["four"] == 0
    assert ref.quantize_block(v, a, select=ref.SEL_FORCE4)["S"] == 0x7C


def _random_blocks(rng, n):
    kinds = rng.integers(0, 4, n)
    out = []
    for k in kinds:
        if k == 0:
            v = rng.standard_normal(16)
        elif k == 1:
            v = rng.standard_t(3, 16)
        elif k == 2:
            v = rng.standard_normal(16) * np.exp(rng.standard_normal(16))
        else:
            v = rng.uniform(-1, 1, 16)
        out.append(v.astype(np.float32))
    return out


def test_selection_invariants_and_forced_modes():
    rng = np.random.default_rng(13)
    n_four = 0
    for v in _random_blocks(rng, 1500):
        alpha = float(np.float32(np.abs(v).max() * rng.uniform(1, 50)) / np.float32(1536.0))
        r = ref.quantize_block(v, alpha)
        r6 = ref.quantize_block(v, alpha, select=ref.SEL_FORCE6)
        r4 = ref.quantize_block(v, alpha, select=ref.SEL_FORCE4)
        assert r["E6"] == r6["E6"] and r["E4"] == r4["E4"]
        assert r["four"] == int(r["E4"] < r["E6"])
        chosen = r4 if r["four"] else r6
        assert r["S"] == chosen["S"] and list(r["codes"]) == list(chosen["codes"])
        assert list(r["D"]) == list(chosen["D"])
        E_chosen = r["E4"] if r["four"] else r["E6"]
        assert E_chosen <= r["E6"]                      # never worse than standard NVFP4
        # recompute the chosen candidate's error in float64 from its outputs
        E64 = float(np.sum((r["D"].astype(np.float64) - v.astype(np.float64)) ** 2))
        assert abs(E64 - E_chosen) <= 1e-5 * max(E64, 1e-30)
        n_four += r["four"]
    assert 100 < n_four < 1400                           # both outcomes occur often


def test_brute_force_over_all_e4m3_scales():
    rng = np.random.default_rng(14)
    for v in _random_blocks(rng, 120):
        alpha = float(np.float32(np.abs(v).max() * 4.0) / np.float32(1536.0))
        r = ref.quantize_block(v, alpha)
        S6 = ref.block_scale(float(np.abs(v).max()), alpha, 6.0)
        S4 = ref.block_scale(float(np.abs(v).max()), alpha, 4.0)
        errs = {S: ref.block_with_scale(v, alpha, S)[0] for S in range(1, 0x7F)}
        best = min(errs.values())
        E_chosen = r["E4"] if r["four"] else r["E6"]
        assert r["S"] in (S4, S6)
        assert errs[S6] == r["E6"] and errs[S4] == r["E4"]
        assert best <= E_chosen <= r["E6"]
        assert E_chosen == min(errs[S4], errs[S6])


def test_rtn_chosen_four_never_uses_code_six():
    # E4M3 rounding moves a normal-range scale by at most 1/16 relatively, so a
    # block mapped to 4 has max|y| <= 4*16/15 < 5 and never rounds up to 6.
    rng = np.random.default_rng(15)
    seen = 0
    for v in _random_blocks(rng, 1500):
        alpha = float(np.float32(np.abs(v).max() * 3.0) / np.float32(1536.0))
        r4 = ref.quantize_block(v, alpha, select=ref.SEL_FORCE4)
        if r4["S"] >= 0x08:                       # normal-range scale
            assert all((c & 7) != 7 for c in r4["codes"])
            seen += 1
        r6 = ref.quantize_block(v, alpha, select=ref.SEL_FORCE6)
        assert max(c & 7 for c in r6["codes"]) >= 6     # the maximum lands on 6 (or 4 after scale rounding)
    assert seen > 1000


def test_figure1_representable_fractions():
    # Mapped to 6, no dequantized magnitude lies strictly between 2/3 of the block
    # maximum and the maximum; mapped to 4, exactly 3/4 of the maximum is available.
    # Use max = 96 with alpha = 1 so that both block scales (16 and 24) are exact.
    top = 96.0
    hit_075 = False
    for t in np.linspace(0.0, top, 769):
        v = [top, float(np.float32(t))]
        d6 = abs(float(ref.quantize_block(v, 1.0, select=ref.SEL_FORCE6)["D"][1]))
        d4 = abs(float(ref.quantize_block(v, 1.0, select=ref.SEL_FORCE4)["D"][1]))
        assert not (top * 2 / 3 < d6 < top)
        if d4 == 0.75 * top:
            hit_075 = True
    assert hit_075
    r = ref.quantize_block([top, 0.75 * top], 1.0)
    assert r["four"] == 1 and r["E4"] == 0.0 and r["E6"] > 0.0
    # Section 3: mapping the maximum to 3 (or 2) only gives subsets of what 6 (or 4) gives
    grid = [Fraction(ref.e2m1_decode(k)) for k in range(8)]
    frac = lambda M: {g / M for g in grid if g <= M}
    assert frac(3) < frac(6) and frac(2) < frac(4)
    assert Fraction(3, 4) in frac(4) and Fraction(3, 4) not in frac(6)
    assert not any(Fraction(2, 3) < f < 1 for f in frac(6))


def test_lossless_on_representable_blocks():
    rng = np.random.default_rng(16)
    for _ in range(200):
        codes = rng.integers(0, 16, 16)
        codes[rng.integers(0, 16)] = 7                   # make the maximum a 6
        S = int(rng.integers(0x20, 0x60))
        alpha = float(2.0 ** rng.integers(-6, 3))
        v = np.array([ref.e2m1_decode(int(c)) for c in codes], np.float32) * np.float32(
            ref.e4m3_decode(S) * alpha)
        r = ref.quantize_block(v, alpha)
        assert r["E6"] == 0.0 and r["four"] == 0 and r["S"] == S
        assert np.array_equal(r["D"], v)
        assert all(int(a) & 7 == int(b) & 7 for a, b in zip(r["codes"], codes))
