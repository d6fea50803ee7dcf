"""Pins for the oracle's NVFP4 x NVFP4 matrix product (the consumer side of Fig. 3)."""
import numpy as np

from oracle import ref
from paper_2512_02010_amd import workloads as wl

E2M1 = np.array([0, .5, 1, 1.5, 2, 3, 4, 6, -0., -.5, -1, -1.5, -2, -3, -4, -6], np.float64)


def _quantized(name, rows, cols, **kw):
    x = wl.bf16_bits(wl.make(name, rows, cols))
    a = ref.tensor_scale(x)
    c, s, _ = ref.quantize(x, a, **kw)
    return x, a, c, s


def _values(codes, scales):
    """a[m][k] = grid(code) * value(scale), written out with numpy from the format definitions
    (Section 1: the E2M1 grid; Section 2.1: E4M3 scales, bias 7, subnormals m * 2^-9)."""
    lo, hi = codes & 15, codes >> 4
    q = np.stack([E2M1[lo], E2M1[hi]], axis=-1).reshape(codes.shape[0], -1)
    e, m = (scales >> 3) & 15, scales & 7
    sv = np.where(e == 0, m * 2.0 ** -9, (1 + m / 8.0) * 2.0 ** (e.astype(np.int64) - 7))
    return q * np.repeat(sv, 16, axis=1)


def test_gemm_equals_float64_matmul_of_the_decoded_operands():
    _, aa, ca, sa = _quantized("c3", 48, 256)
    _, ab, cb, sb = _quantized("c2", 80, 256)
    A, Bm = _values(ca, sa), _values(cb, sb)
    want = (np.float64(np.float32(aa)) * np.float64(np.float32(ab))) * (A @ Bm.T)
    got, got_abs = ref.gemm(ca, sa, aa, cb, sb, ab, want_abs=True)
    assert got.shape == (48, 80)
    # both are fp64 sums of the same exact products, only the order differs
    assert np.allclose(got, want, rtol=0, atol=1e-12 * np.abs(want).max())
    want_abs = (np.float64(np.float32(aa)) * np.float64(np.float32(ab))) * (np.abs(A) @ np.abs(Bm).T)
    assert np.allclose(got_abs, want_abs, rtol=1e-12)
    assert (got_abs >= np.abs(got) * (1 - 1e-12)).all()


def test_gemm_decoded_operands_equal_the_pinned_dequantizer():
    # value(code) * value(scale) is exact in BF16 (6 significant bits), so the dequantizer with
    # alpha = 1 returns exactly the operand values the product is defined on
    _, _, c, s = _quantized("c5", 32, 128)
    d = ref.dequantize(c, s, 1.0, 32, 128)
    assert np.array_equal((d.astype(np.uint32) << 16).view(np.float32).astype(np.float64),
                          _values(c, s))


def test_gemm_closed_forms():
    K = 64
    ones_codes = np.full((3, K // 2), 0x22, np.uint8)          # every element 1.0
    unit_scale = np.full((3, K // 16), 0x38, np.uint8)         # E4M3 1.0
    # all ones: C = alpha_a * alpha_b * K
    got = ref.gemm(ones_codes, unit_scale, 0.5, ones_codes, unit_scale, 0.25)
    assert np.array_equal(got, np.full((3, 3), 0.5 * 0.25 * K))
    # a one-hot row picks one element of the other operand, scale included
    _, _, cb, sb = _quantized("c1", 5, K)
    Bv = _values(cb, sb)
    ca = np.zeros((K, K // 2), np.uint8)
    for k in range(K):
        ca[k, k // 2] = 0x2 << (4 * (k & 1))                   # 1.0 at position k
    sa = np.full((K, K // 16), 0x40, np.uint8)                 # E4M3 2.0
    got = ref.gemm(ca, sa, 1.0, cb, sb, 1.0)
    assert np.array_equal(got, 2.0 * Bv.T)
    # signs: -1.5 * 1.5 summed over a block of 16 with scales 0.5 and 4
    ca = np.full((1, 8), 0xBB, np.uint8)
    cb = np.full((1, 8), 0x33, np.uint8)
    got = ref.gemm(ca, np.array([[0x30]], np.uint8), 1.0, cb, np.array([[0x48]], np.uint8), 1.0)
    assert got[0, 0] == 16 * (-1.5 * 0.5) * (1.5 * 4.0)


def test_gemm_symmetry_and_block_scale_linearity():
    _, aa, ca, sa = _quantized("c1", 24, 128)
    _, ab, cb, sb = _quantized("c4", 40, 128)
    got = ref.gemm(ca, sa, aa, cb, sb, ab)
    assert np.array_equal(ref.gemm(cb, sb, ab, ca, sa, aa), got.T)
    # halving every scale of A (exponent field - 1, all of them normal with room) halves C
    assert (sa >= 16).all()
    assert np.array_equal(ref.gemm(ca, (sa - 8).astype(np.uint8), aa, cb, sb, ab), 0.5 * got)
    # zeroing one k-block of A removes exactly that block's contribution
    sa0 = sa.copy()
    sa0[:, 3] = 0
    part = ref.gemm(ca[:, 24:32].copy(), sa[:, 3:4].copy(), aa, cb[:, 24:32].copy(),
                    sb[:, 3:4].copy(), ab)
    assert np.allclose(ref.gemm(ca, sa0, aa, cb, sb, ab), got - part, rtol=0,
                       atol=1e-12 * np.abs(got).max())


def test_quantized_product_approximates_the_bf16_product():
    """End to end: the product of the two 4/6-quantized operands is the product of the
    original tensors up to quantization noise, and 4/6 is no worse than scaling to 6 only."""
    xa = wl.make("c1", 64, 512)
    xb_ = wl.make("c4", 96, 512)
    exact = xa.double().numpy() @ xb_.double().numpy().T
    errs = {}
    for sel in (ref.SEL_46_MSE, ref.SEL_FORCE6):
        ops = []
        for x in (xa, xb_):
            bits = wl.bf16_bits(x)
            a = ref.tensor_scale(bits)
            c, s, _ = ref.quantize(bits, a, select=sel)
            ops += [c, s, a]
        got = ref.gemm(*ops)
        errs[sel] = float(np.sqrt(((got - exact) ** 2).mean()) / np.sqrt((exact ** 2).mean()))
    assert errs[ref.SEL_46_MSE] < 0.2 and errs[ref.SEL_FORCE6] < 0.2
    assert errs[ref.SEL_46_MSE] < errs[ref.SEL_FORCE6]


def test_gemm_with_tile_scales_equals_gemm_with_the_scales_repeated_per_row():
    """An operand quantized with 16x16 tiles carries one scale line per 16 rows; using it is
    the same as repeating every line sixteen times."""
    xw = wl.bf16_bits(wl.make("c2", 64, 128))
    aw = ref.tensor_scale(xw)
    cw, sw, _, _ = ref.quantize_2d(xw, aw)
    _, ax, cx, sx = _quantized("c3", 40, 128)
    got = ref.gemm(cx, sx, ax, cw, sw, aw, tiles_b=True)
    want = ref.gemm(cx, sx, ax, cw, np.repeat(sw, 16, axis=0), aw)
    assert np.array_equal(got, want)
    assert np.array_equal(ref.gemm(cw, sw, aw, cx, sx, ax, tiles_a=True), want.T)
    # the transposed packing multiplies from the other side: W^T [128][64] against a [24][64] operand
    cc, sc, _ = ref.repack_2d_columnwise(cw, sw, np.zeros_like(sw))
    _, ag, cg, sg = _quantized("c1", 24, 64)
    got_t = ref.gemm(cg, sg, ag, cc, sc, aw, tiles_b=True)
    w_deq = (ref.dequantize_2d(cw, sw, 1.0, 64, 128).astype(np.uint32) << 16).view(np.float32)
    g_val = _values(cg, sg)
    want_t = np.float64(np.float32(ag)) * np.float64(np.float32(aw)) * (g_val @ w_deq.astype(np.float64))
    assert np.allclose(got_t, want_t, rtol=0, atol=1e-12 * np.abs(want_t).max())
