"""Pins for the oracle's fp32-input entry points (FP32 master weights entering the quantizer
directly, Fig. 3).  The per-block procedure is pinned elsewhere on fp32 values; here the
tensor-level fetch, layouts and packing are tied to it, and to the BF16-input path wherever the
two must coincide."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2512_02010_amd import workloads as wl

SR_SEED, RHT_SEED = wl.C5_SR_SEED, wl.C5_RHT_SEED


def _pair(name, rows, cols):
    """The same BF16-representable values as BF16 bit patterns and as an fp32 array."""
    x = wl.make(name, rows, cols)
    return wl.bf16_bits(x), x.float().numpy()


@pytest.mark.parametrize("layout", [ref.ROWWISE, ref.COLWISE])
@pytest.mark.parametrize("rounding,rht", [(ref.RTN, 0), (ref.SR, 0), (ref.RTN, 1), (ref.SR, 1),
                                          (ref.SR_AFTER_RTN_SELECT, 0)])
def test_bf16_representable_values_give_the_bf16_results(layout, rounding, rht):
    xb, xf = _pair("c3", 48, 160)
    kw = dict(layout=layout, rht=rht, rht_seed=RHT_SEED)
    a = ref.tensor_scale(xb, **kw)
    assert ref.tensor_scale(xf, **kw) == a
    kw.update(rounding=rounding, sr_seed=SR_SEED, want_deq=True)
    for got, want in zip(ref.quantize(xf, a, **kw), ref.quantize(xb, a, **kw)):
        assert np.array_equal(got, want)
    kw.pop("want_deq")
    assert np.array_equal(ref.fake_quant(xf, a, **kw), ref.fake_quant(xb, a, **kw))


def test_bf16_representable_values_2d_blocks():
    xb, xf = _pair("c2", 64, 96)
    a = ref.tensor_scale(xb)
    for sel in (ref.SEL_46_MSE, ref.SEL_46_MAE):
        for got, want in zip(ref.quantize_2d(xf, a, select=sel), ref.quantize_2d(xb, a, select=sel)):
            assert np.array_equal(got, want)


def test_fp32_tensor_equals_the_per_block_procedure_on_unrounded_values():
    x = wl.make("c2", 32, 128, dtype=torch.float32).numpy()
    # the draws are genuinely fp32: most are not BF16 values
    assert (x.view(np.uint32) & 0xFFFF != 0).mean() > 0.9
    alpha = ref.tensor_scale(x)
    assert alpha == float(np.float32(np.abs(x).max()) / np.float32(1536.0))
    codes, scales, choice, deq = ref.quantize(x, alpha, want_deq=True)
    for r in (0, 5, 31):
        for b in range(8):
            blk = ref.quantize_block(x[r, 16 * b:16 * b + 16], alpha)
            assert scales[r, b] == blk["S"] and choice[r, b] == blk["four"]
            packed = codes[r, 8 * b:8 * b + 8]
            assert list(packed & 15) == list(blk["codes"][0::2])
            assert list(packed >> 4) == list(blk["codes"][1::2])
            want = [ref.f32_to_bf16(float(d)) for d in blk["D"]]
            assert list(deq[r, 16 * b:16 * b + 16]) == want
    assert np.array_equal(ref.dequantize(codes, scales, alpha, 32, 128), deq)


def test_fp32_input_is_not_rounded_to_bf16_on_the_way_in():
    """Quantizing the fp32 values and quantizing their BF16 roundings must differ somewhere:
    the block maximum (hence the scale byte) and near-midpoint elements see the low bits."""
    xf = wl.make("c2", 128, 256, dtype=torch.float32)
    xr = wl.bf16_bits(xf.to(torch.bfloat16))
    x = xf.numpy()
    alpha = ref.tensor_scale(x)
    c32, s32, _ = ref.quantize(x, alpha)
    c16, s16, _ = ref.quantize(xr, alpha)
    assert (c32 != c16).any() and (s32 != s16).any()
    # yet the two stay close: with the choice taken out (always 6) a block's scale moves by at
    # most one E4M3 step
    _, s32, _ = ref.quantize(x, alpha, select=ref.SEL_FORCE6)
    _, s16, _ = ref.quantize(xr, alpha, select=ref.SEL_FORCE6)
    assert (s32 != s16).any() and np.abs(s32.astype(int) - s16.astype(int)).max() <= 1


@pytest.mark.parametrize("rounding", [ref.RTN, ref.SR])
def test_fp32_columnwise_is_rowwise_of_the_transpose(rounding):
    x = wl.make("c4", 48, 160, dtype=torch.float32).numpy()
    xt = np.ascontiguousarray(x.T)
    alpha = ref.tensor_scale(x)
    assert ref.tensor_scale(x, layout=ref.COLWISE) == alpha
    c_col, s_col, f_col, d_col = ref.quantize(x, alpha, layout=ref.COLWISE, want_deq=True)
    c_row, s_row, f_row, d_row = ref.quantize(xt, alpha, layout=ref.ROWWISE, want_deq=True)
    assert np.array_equal(c_col, c_row) and np.array_equal(s_col, s_row)
    assert np.array_equal(f_col, f_row) and np.array_equal(d_col, d_row.T)
    if rounding == ref.SR:
        # stochastic rounding is keyed by the element's flat index in x, so it is NOT the
        # rowwise result of the transposed tensor; tie it to the per-block procedure instead
        c, s, f = ref.quantize(x, alpha, layout=ref.COLWISE, rounding=ref.SR, sr_seed=SR_SEED)
        col, blk = 7, 2
        v = x[16 * blk:16 * blk + 16, col]
        u = [ref.sr_uniform(SR_SEED, (16 * blk + i) * 160 + col) for i in range(16)]
        want = ref.quantize_block(v, alpha, rounding=ref.SR, u=u)
        assert s[col, blk] == want["S"] and f[col, blk] == want["four"]
        packed = c[col, 8 * blk:8 * blk + 8]
        assert list(packed & 15) == list(want["codes"][0::2])
        assert list(packed >> 4) == list(want["codes"][1::2])


def test_fp32_2d_blocks_share_the_tile_scale():
    x = wl.make("c2", 64, 96, dtype=torch.float32).numpy()
    alpha = ref.tensor_scale(x)
    codes, scales, choice, deq = ref.quantize_2d(x, alpha)
    assert scales.shape == (4, 6)
    for tr, tc in ((0, 0), (3, 5), (2, 1)):
        tile = x[16 * tr:16 * tr + 16, 16 * tc:16 * tc + 16]
        b = float(np.abs(tile).max())
        S = ref.block_scale(b, alpha, 4.0 if choice[tr, tc] else 6.0)
        assert scales[tr, tc] == S
        for r in range(16):
            _, q, D = ref.block_with_scale(tile[r], alpha, S)
            packed = codes[16 * tr + r, 8 * tc:8 * tc + 8]
            assert list(packed & 15) == list(q[0::2]) and list(packed >> 4) == list(q[1::2])
    assert np.array_equal(ref.dequantize_2d(codes, scales, alpha, 64, 96), deq)
