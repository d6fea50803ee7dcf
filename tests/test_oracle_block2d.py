"""Pins for the oracle's 2D (16x16-tile) block quantization (named in Section 4.1)."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import ref
from paper_2512_02010_amd import workloads as wl


def _f32(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


def _tile(xf, tr, tc):
    return xf[16 * tr:16 * tr + 16, 16 * tc:16 * tc + 16]


def test_tile_scale_rows_and_packing():
    x = wl.bf16_bits(wl.make("c2", 64, 96))
    xf = _f32(x)
    alpha = ref.tensor_scale(x)
    for sel in (ref.SEL_FORCE6, ref.SEL_FORCE4):
        codes, scales, choice, deq = ref.quantize_2d(x, alpha, select=sel)
        M = 6.0 if sel == ref.SEL_FORCE6 else 4.0
        for tr, tc in ((0, 0), (1, 3), (3, 5)):
            t = _tile(xf, tr, tc)
            S = ref.block_scale(float(np.abs(t).max()), alpha, M)        # one scale per tile
            assert scales[tr, tc] == S and choice[tr, tc] == (sel == ref.SEL_FORCE4)
            for r in range(16):
                E, q, D = ref.block_with_scale(t[r], alpha, S)            # rows share it
                packed = codes[16 * tr + r, 8 * tc:8 * tc + 8]
                assert list(packed & 15) == list(q[0::2]) and list(packed >> 4) == list(q[1::2])
                want = np.array([ref.f32_to_bf16(float(d)) for d in D], np.uint16)
                assert np.array_equal(deq[16 * tr + r, 16 * tc:16 * tc + 16], want)
        assert np.array_equal(ref.dequantize_2d(codes, scales, alpha, 64, 96), deq)


@pytest.mark.parametrize("sel", [ref.SEL_46_MSE, ref.SEL_46_MAE, ref.SEL_46_ABSMAX])
def test_tile_selection_is_by_the_tile_error(sel):
    x = wl.bf16_bits(wl.make("c3", 96, 128))
    xf = _f32(x)
    alpha = ref.tensor_scale(x)
    codes, scales, choice, deq = ref.quantize_2d(x, alpha, select=sel)
    c6, s6, _, d6 = ref.quantize_2d(x, alpha, select=ref.SEL_FORCE6)
    c4, s4, _, d4 = ref.quantize_2d(x, alpha, select=ref.SEL_FORCE4)
    n4 = 0
    for tr in range(6):
        for tc in range(8):
            t = _tile(xf, tr, tc).astype(np.float64)
            e6 = np.abs(_tile(_f32(d6), tr, tc).astype(np.float64) - t)
            e4 = np.abs(_tile(_f32(d4), tr, tc).astype(np.float64) - t)
            # BF16 output rounding is far below the FP4 error; compare the metrics in fp64
            m = {ref.SEL_46_MSE: lambda e: (e ** 2).sum(), ref.SEL_46_MAE: lambda e: e.sum(),
                 ref.SEL_46_ABSMAX: lambda e: e.max()}[sel]
            if abs(m(e4) - m(e6)) > 2e-2 * max(m(e4), m(e6)):
                assert choice[tr, tc] == int(m(e4) < m(e6)), (tr, tc)
            src_c, src_s = (c4, s4) if choice[tr, tc] else (c6, s6)
            assert scales[tr, tc] == src_s[tr, tc]
            assert np.array_equal(codes[16 * tr:16 * tr + 16, 8 * tc:8 * tc + 8],
                                  src_c[16 * tr:16 * tr + 16, 8 * tc:8 * tc + 8])
            n4 += choice[tr, tc]
    assert 0 < n4 < 48


def test_tile_error_order_on_exact_inputs():
    """Few-bit inputs, alpha = 1: every fp32 operation is exact, so the tile decision must
    equal the decision on exact rational sums (any summation order gives the same)."""
    rng = np.random.default_rng(61)
    flips = 0
    for _ in range(40):
        t = (rng.integers(-24, 25, (16, 16)) * 0.25).astype(np.float32)
        t[rng.integers(0, 16), rng.integers(0, 16)] = 6.0
        bits = np.array([[ref.f32_to_bf16(float(v)) for v in row] for row in t], np.uint16)
        codes, scales, choice, deq = ref.quantize_2d(bits, 1.0)
        E = {}
        for name, M in (("6", 6.0), ("4", 4.0)):
            S = ref.block_scale(6.0, 1.0, M)
            E[name] = sum(Fraction(ref.block_with_scale(t[r], 1.0, S)[0]) for r in range(16))
        assert choice[0, 0] == int(E["4"] < E["6"])
        flips += choice[0, 0]
    assert 0 < flips < 40


def test_a_matrix_and_its_transpose_get_the_same_tiles_under_a_fixed_scale_rule():
    # the point of 2D blocks: with one scale per 16x16 tile, quantizing W^T gives the
    # transpose of quantizing W (same scales, same values)
    x = wl.bf16_bits(wl.make("c4", 64, 96))
    xt = np.ascontiguousarray(x.T)
    alpha = ref.tensor_scale(x)
    for sel in (ref.SEL_FORCE6, ref.SEL_FORCE4):
        _, s, _, d = ref.quantize_2d(x, alpha, select=sel)
        _, st, _, dt = ref.quantize_2d(xt, alpha, select=sel)
        assert np.array_equal(st, s.T) and np.array_equal(dt, d.T)
    # 1x16 blocks do not have this property
    d_row = ref.fake_quant(x, alpha, select=ref.SEL_FORCE6)
    d_row_t = ref.fake_quant(xt, alpha, select=ref.SEL_FORCE6)
    assert not np.array_equal(d_row_t, d_row.T)


def test_2d_with_stochastic_rounding_modes():
    x = wl.bf16_bits(wl.make("c5", 32, 64))
    alpha = ref.tensor_scale(x)
    seed = wl.C5_SR_SEED
    xf = _f32(x)
    c_sr, s_sr, f_sr, _ = ref.quantize_2d(x, alpha, rounding=ref.SR, sr_seed=seed)
    c_mix, s_mix, f_mix, _ = ref.quantize_2d(x, alpha, rounding=ref.SR_AFTER_RTN_SELECT, sr_seed=seed)
    _, s_rtn, f_rtn, _ = ref.quantize_2d(x, alpha)
    assert np.array_equal(s_mix, s_rtn) and np.array_equal(f_mix, f_rtn)
    tr, tc, r = 1, 2, 5
    row = 16 * tr + r
    u = np.array([ref.sr_uniform(seed, row * 64 + 16 * tc + i) for i in range(16)], np.float32)
    for codes, scales in ((c_sr, s_sr), (c_mix, s_mix)):
        E, q, D = ref.block_with_scale(xf[row, 16 * tc:16 * tc + 16], alpha, int(scales[tr, tc]),
                                       ref.SR, u)
        packed = codes[row, 8 * tc:8 * tc + 8]
        assert list(packed & 15) == list(q[0::2]) and list(packed >> 4) == list(q[1::2])


def test_columnwise_packing_of_2d_blocks_is_the_transposed_matrix():
    """The tiles are decided once; W^T gets the same codes and scales packed along its rows."""
    x = wl.bf16_bits(wl.make("c2", 64, 96))
    alpha = ref.tensor_scale(x)
    codes, scales, choice, deq = ref.quantize_2d(x, alpha)
    cc, sc, fc = ref.repack_2d_columnwise(codes, scales, choice)
    assert cc.shape == (96, 32) and sc.shape == (6, 4)
    # nibble by nibble: code of element (r, c)
    lo, hi = codes & 15, codes >> 4
    q = np.stack([lo, hi], axis=-1).reshape(64, 96)
    qt = np.stack([cc & 15, cc >> 4], axis=-1).reshape(96, 64)
    assert np.array_equal(qt, q.T)
    assert np.array_equal(sc, scales.T) and np.array_equal(fc, choice.T)
    # both packings dequantize to the same matrix
    assert np.array_equal(ref.dequantize_2d_columnwise(cc, sc, alpha, 64, 96), deq)
    # and it is what a rowwise-packed dequantizer makes of W^T
    assert np.array_equal(ref.dequantize_2d(cc, sc, alpha, 96, 64), deq.T)
    # under a fixed scale rule nothing depends on the order of the error sums, so this equals
    # quantizing the transposed matrix outright
    c6, s6, f6, _ = ref.quantize_2d(x, alpha, select=ref.SEL_FORCE6)
    ct, st, ft, _ = ref.quantize_2d(np.ascontiguousarray(x.T), alpha, select=ref.SEL_FORCE6)
    cc6, sc6, fc6 = ref.repack_2d_columnwise(c6, s6, f6)
    assert np.array_equal(cc6, ct) and np.array_equal(sc6, st) and np.array_equal(fc6, ft)
