"""Pins for the oracle's whole-tensor entry points (layouts, packing, round trips)."""
import numpy as np
import pytest

from oracle import ref
from paper_2512_02010_amd import workloads as wl


def _small(name, rows, cols):
    return wl.bf16_bits(wl.make(name, rows, cols))


def _f32(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


def test_tensor_scale_is_eq1_with_256_or_448():
    x = _small("c1", 64, 256)
    amax = np.float32(np.abs(_f32(x)).max())
    assert ref.tensor_scale(x) == float(amax / np.float32(1536.0))
    assert ref.tensor_scale(x, fp8_max=448.0) == float(amax / np.float32(2688.0))
    assert ref.tensor_scale(x, layout=ref.COLWISE) == ref.tensor_scale(x)
    z = np.zeros((16, 32), np.uint16)
    assert ref.tensor_scale(z) == 1.0
    z[:] = 0x8000                                  # all -0.0
    assert ref.tensor_scale(z) == 1.0


def test_quantize_equals_per_block_procedure_and_packing():
    x = _small("c2", 32, 128)
    alpha = ref.tensor_scale(x)
    codes, scales, choice = ref.quantize(x, alpha)
    assert codes.shape == (32, 64) and scales.shape == (32, 8) and choice.shape == (32, 8)
    xf = _f32(x)
    for r in (0, 7, 31):
        for b in range(8):
            blk = ref.quantize_block(xf[r, 16 * b:16 * b + 16], alpha)
            assert scales[r, b] == blk["S"] and choice[r, b] == blk["four"]
            packed = codes[r, 8 * b:8 * b + 8]
            # even element in the low nibble, odd element in the high nibble
            assert list(packed & 15) == list(blk["codes"][0::2])
            assert list(packed >> 4) == list(blk["codes"][1::2])
    assert set(np.unique(choice)) <= {0, 1} and 0 < choice.mean() < 1


@pytest.mark.parametrize("name", ["c1", "c3", "c4"])
def test_columnwise_is_rowwise_of_the_transpose(name):
    x = _small(name, 48, 160)
    xt = np.ascontiguousarray(x.T)
    alpha = ref.tensor_scale(x)
    c_col, s_col, f_col, d_col = ref.quantize(x, alpha, layout=ref.COLWISE, want_deq=True)
    c_row, s_row, f_row, d_row = ref.quantize(xt, alpha, layout=ref.ROWWISE, want_deq=True)
    assert c_col.shape == (160, 24) and s_col.shape == (160, 3)
    assert np.array_equal(c_col, c_row) and np.array_equal(s_col, s_row)
    assert np.array_equal(f_col, f_row)
    assert np.array_equal(d_col, d_row.T)          # output stays in x's own orientation


@pytest.mark.parametrize("layout", [ref.ROWWISE, ref.COLWISE])
@pytest.mark.parametrize("select", [ref.SEL_46_MSE, ref.SEL_FORCE6, ref.SEL_FORCE4])
def test_dequantize_of_quantize_equals_fake_quant(layout, select):
    x = _small("c3", 64, 96)
    alpha = ref.tensor_scale(x, layout=layout)
    codes, scales, choice, deq = ref.quantize(x, alpha, layout=layout, select=select, want_deq=True)
    out = ref.dequantize(codes, scales, alpha, 64, 96, layout=layout)
    fq = ref.fake_quant(x, alpha, layout=layout, select=select)
    assert np.array_equal(out, fq) and np.array_equal(out, deq)
    # dequantize is value(code) * (value(scale) * alpha), cast to BF16
    xf = _f32(out)
    r, c = 5, 37
    if layout == ref.ROWWISE:
        byte, S = codes[r, c // 2], scales[r, c // 16]
        code = (byte >> 4) if c & 1 else (byte & 15)
    else:
        byte, S = codes[c, r // 2], scales[c, r // 16]
        code = (byte >> 4) if r & 1 else (byte & 15)
    want = np.float32(ref.e2m1_decode(int(code))) * (np.float32(ref.e4m3_decode(int(S))) * np.float32(alpha))
    assert xf[r, c] == _f32(np.array([ref.f32_to_bf16(float(want))], np.uint16))[0]


def test_quantizing_a_dequantized_tensor_is_lossless():
    x = _small("c1", 32, 64)
    alpha = ref.tensor_scale(x)
    fq = ref.fake_quant(x, alpha, select=ref.SEL_FORCE6)
    # powers of two keep fq representable in BF16 only if few bits: re-quantize
    # the BF16 result and require a fixed point after one more round
    fq2 = ref.fake_quant(fq, alpha, select=ref.SEL_FORCE6)
    fq3 = ref.fake_quant(fq2, alpha, select=ref.SEL_FORCE6)
    assert np.array_equal(fq2, fq3)


def test_choice_invariants_on_tensor():
    x = _small("c2", 64, 256)
    alpha = ref.tensor_scale(x)
    E6, E4 = ref.block_errors(x, alpha)
    _, _, choice = ref.quantize(x, alpha)
    assert np.array_equal(choice.astype(bool), E4 < E6)
    chosen = np.where(choice.astype(bool), E4, E6)
    assert np.all(chosen <= E6)


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c5"])
def test_tensor_mse_four_over_six_not_worse_than_force6(name):
    x = _small(name, 128, 256)
    alpha = ref.tensor_scale(x)
    xf = _f32(x).astype(np.float64)
    mse = {}
    for sel in (ref.SEL_46_MSE, ref.SEL_FORCE6, ref.SEL_FORCE4):
        d = _f32(ref.fake_quant(x, alpha, select=sel)).astype(np.float64)
        mse[sel] = np.mean((d - xf) ** 2)
    # BF16 output rounding is far below the FP4 error, so the per-block
    # guarantee carries over to the tensor
    assert mse[ref.SEL_46_MSE] <= mse[ref.SEL_FORCE6] * (1 + 1e-3)
    assert mse[ref.SEL_46_MSE] <= mse[ref.SEL_FORCE4] * (1 + 1e-3)


def test_sr_tensor_uses_flat_element_index():
    x = _small("c5", 32, 64)
    seed = wl.C5_SR_SEED
    alpha = ref.tensor_scale(x)
    xf = _f32(x)
    for layout in (ref.ROWWISE, ref.COLWISE):
        codes, scales, choice = ref.quantize(x, alpha, layout=layout, rounding=ref.SR, sr_seed=seed)
        for line, blk in ((0, 0), (3, 1), (31, 1)):
            if layout == ref.ROWWISE:
                idx = [(line, 16 * blk + i) for i in range(16)]
            else:
                idx = [(16 * blk + i, line) for i in range(16)]
            v = np.array([xf[r, c] for r, c in idx], np.float32)
            u = np.array([ref.sr_uniform(seed, r * 64 + c) for r, c in idx], np.float32)
            b = ref.quantize_block(v, alpha, ref.SR, ref.SEL_46_MSE, u)
            assert scales[line, blk] == b["S"] and choice[line, blk] == b["four"]
            packed = codes[line, 8 * blk:8 * blk + 8]
            assert list(packed & 15) == list(b["codes"][0::2])
            assert list(packed >> 4) == list(b["codes"][1::2])
    # RTN and SR differ, and two seeds differ
    c_rtn, _, _ = ref.quantize(x, alpha)
    c_sr, _, _ = ref.quantize(x, alpha, rounding=ref.SR, sr_seed=seed)
    c_sr2, _, _ = ref.quantize(x, alpha, rounding=ref.SR, sr_seed=seed + 1)
    assert not np.array_equal(c_rtn, c_sr) and not np.array_equal(c_sr, c_sr2)


def test_rht_tensor_path():
    x = _small("c5", 32, 96)
    seed = wl.C5_RHT_SEED
    xf = _f32(x)
    # the tensor scale is taken over the transformed values
    vmax = 0.0
    for r in range(32):
        for b in range(6):
            y = ref.rht16(xf[r, 16 * b:16 * b + 16], ref.rht_sign_word(seed, b))
            vmax = max(vmax, float(np.abs(y).max()))
    alpha = ref.tensor_scale(x, rht=1, rht_seed=seed)
    assert alpha == float(np.float32(vmax) / np.float32(1536.0))
    codes, scales, choice, deq = ref.quantize(x, alpha, rht=1, rht_seed=seed, want_deq=True)
    for r, b in ((0, 0), (17, 5)):
        y = ref.rht16(xf[r, 16 * b:16 * b + 16], ref.rht_sign_word(seed, b))
        blk = ref.quantize_block(y, alpha)
        assert scales[r, b] == blk["S"] and choice[r, b] == blk["four"]
        got = _f32(deq[r, 16 * b:16 * b + 16])
        want = _f32(np.array([ref.f32_to_bf16(float(d)) for d in blk["D"]], np.uint16))
        assert np.array_equal(got, want)         # result stays in the transformed domain
    # columnwise: the sign word depends on the block position along the rows
    xt = np.ascontiguousarray(x.T)               # 96 x 32
    a_c = ref.tensor_scale(xt, layout=ref.COLWISE, rht=1, rht_seed=seed)
    a_r = ref.tensor_scale(x, layout=ref.ROWWISE, rht=1, rht_seed=seed)
    assert a_c == a_r
    cc = ref.quantize(xt, a_c, layout=ref.COLWISE, rht=1, rht_seed=seed)
    cr = ref.quantize(x, a_r, layout=ref.ROWWISE, rht=1, rht_seed=seed)
    assert all(np.array_equal(p, q) for p, q in zip(cc, cr))


def test_workload_generators_are_deterministic_and_shaped():
    for name in ("c1", "c2", "c3", "c4", "c5"):
        a = wl.bf16_bits(wl.make(name, 32, 64))
        b = wl.bf16_bits(wl.make(name, 32, 64))
        assert a.shape == (32, 64) and np.array_equal(a, b)
        assert np.isfinite(_f32(a)).all()
    x2 = _f32(wl.bf16_bits(wl.make("c2", 64, 512)))
    col_energy = np.abs(x2).mean(axis=0)
    assert (col_energy > 10 * np.median(col_energy)).sum() == 5      # 1 % of 512 columns
    x3 = _f32(wl.bf16_bits(wl.make("c3", 256, 512)))
    frac = (np.abs(x3) >= 100).mean()
    assert 2e-4 < frac < 3e-3
    for kind in wl.ADVERSARIAL_KINDS:
        t = wl.adversarial(kind)
        assert t.shape == (32, 64)


@pytest.mark.parametrize("layout", [ref.ROWWISE, ref.COLWISE])
def test_quantizing_a_slice_of_rows_gives_that_slice_of_the_whole(layout):
    x = _small("c5", 96, 160)
    alpha = ref.tensor_scale(x)
    kw = dict(layout=layout, rounding=ref.SR, rht=1, sr_seed=wl.C5_SR_SEED, rht_seed=wl.C5_RHT_SEED)
    c, s, f, d = ref.quantize(x, alpha, want_deq=True, **kw)
    r0, n = 32, 48
    cs, ss, fs, ds = ref.quantize_rows(np.ascontiguousarray(x[r0:r0 + n]), r0, alpha, **kw)
    assert np.array_equal(ds, d[r0:r0 + n])
    if layout == ref.ROWWISE:
        assert np.array_equal(cs, c[r0:r0 + n]) and np.array_equal(ss, s[r0:r0 + n])
        assert np.array_equal(fs, f[r0:r0 + n])
    else:
        assert np.array_equal(cs, c[:, r0 // 2:(r0 + n) // 2])
        assert np.array_equal(ss, s[:, r0 // 16:(r0 + n) // 16])
    # with the offset left out the random numbers differ, so the slice would not match
    c0, _, _, _ = ref.quantize_rows(np.ascontiguousarray(x[r0:r0 + n]), 0, alpha, **kw)
    assert not np.array_equal(c0, cs)
