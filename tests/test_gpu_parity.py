"""GPU: the HIP library against the CPU oracle, element by element, through the C ABI.

Bar: codes, scale bytes, per-block 4-vs-6 choices and the tensor scale are bit-exact;
dequantized / fake-quantized BF16 values are identical to 0 ULP (compared as bit
patterns, so the sign of zero counts too)."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2512_02010_amd import binding as B
from paper_2512_02010_amd import workloads as wl

pytestmark = pytest.mark.gpu

SR_SEED, RHT_SEED = wl.C5_SR_SEED, wl.C5_RHT_SEED


def _log(msg):
    print(msg, flush=True)


def _np(t):
    return None if t is None else t.cpu().numpy()


def _bits(t):
    return t.cpu().view(torch.int16).numpy().view(np.uint16)


def _alpha_bits(a):
    return np.array([a], np.float32).view(np.uint32)[0]


_WS = None


def _workspace():
    """One workspace for all cases: each call must leave it zeroed for the next."""
    global _WS
    if _WS is None:
        _WS = B.new_workspace()
    return _WS


def check_case(x: torch.Tensor, layout=B.ROWWISE, rounding=B.RTN, select=B.SEL_46_MSE, rht=0,
               fp8_max=256.0, alpha_value=None, tag=""):
    """Run tensor_scale -> quantize -> dequantize -> fake_quant on the GPU and compare every
    output with the oracle on the same bits."""
    rows, cols = x.shape
    _log(f"case {tag} shape={rows}x{cols} layout={layout} rounding={rounding} select={select} "
         f"rht={rht} fp8_max={fp8_max}")
    xb = wl.host_array(x)          # BF16 bit patterns, or the fp32 values themselves
    xd = x.cuda()
    kw = dict(rounding=rounding, select=select, rht=rht, sr_seed=SR_SEED, rht_seed=RHT_SEED)
    layouts = [l for l in (B.ROWWISE, B.COLWISE) if layout & l]

    # tensor scale (one orientation at a time; without the transform both agree)
    alphas = {}
    for l in layouts:
        a_ref = ref.tensor_scale(xb, layout=l, rht=rht, rht_seed=RHT_SEED, fp8_max=fp8_max)
        a_gpu = B.nvfp4_46_tensor_scale(xd, layout=l, rht=rht, rht_seed=RHT_SEED, fp8_max=fp8_max)
        assert _alpha_bits(a_gpu.item()) == _alpha_bits(a_ref), (tag, l, a_gpu.item(), a_ref)
        # the one-launch form, on a workspace that every case of this module shares
        a_ws = B.nvfp4_46_tensor_scale_ws(xd, _workspace(), layout=l, rht=rht, rht_seed=RHT_SEED,
                                          fp8_max=fp8_max)
        assert _alpha_bits(a_ws.item()) == _alpha_bits(a_ref), (tag, l, "ws", a_ws.item(), a_ref)
        alphas[l] = a_gpu
    if alpha_value is not None:
        alphas = {l: torch.tensor([alpha_value], dtype=torch.float32, device="cuda") for l in layouts}
    alpha = alphas[layouts[0]]
    a_host = float(alpha.item())
    if len(layouts) == 2:
        assert _alpha_bits(alphas[B.ROWWISE].item()) == _alpha_bits(alphas[B.COLWISE].item())

    out = B.nvfp4_46_quantize(xd, alpha, layout=layout, fp8_max=fp8_max, **kw)
    torch.cuda.synchronize()
    for l in layouts:
        sfx = "row" if l == B.ROWWISE else "col"
        c_ref, s_ref, f_ref, d_ref = ref.quantize(xb, a_host, layout=l, want_deq=True, **kw)
        for name, want in (("scales", s_ref), ("choice", f_ref), ("codes", c_ref)):
            got = _np(out[f"{name}_{sfx}"])
            if not np.array_equal(got, want):
                bad = np.argwhere(got != want)
                raise AssertionError(f"{tag}: {name}_{sfx} differs at {len(bad)} places, first "
                                     f"{bad[:4].tolist()} gpu {got[tuple(bad[0])]} "
                                     f"oracle {want[tuple(bad[0])]}")
        deq = B.nvfp4_46_dequantize(out[f"codes_{sfx}"], out[f"scales_{sfx}"], alpha, rows, cols,
                                    layout=l)
        assert np.array_equal(_bits(deq), d_ref), f"{tag}: dequantize_{sfx}"
        assert np.array_equal(ref.dequantize(c_ref, s_ref, a_host, rows, cols, layout=l), d_ref)
        fq = B.nvfp4_46_fake_quant(xd, alpha, layout=l, fp8_max=fp8_max, **kw)
        assert np.array_equal(_bits(fq), d_ref), f"{tag}: fake_quant_{sfx}"
    return out


# ------------------------------------------------------------------ small, many options

SHAPES_ROW = [(16, 16), (48, 176), (144, 272), (1, 4096), (257, 48), (1000, 4112)]
SHAPES_COL = [(16, 8), (48, 176), (144, 264), (272, 136), (4096, 8), (128, 128), (1008, 4104)]


@pytest.mark.parametrize("shape", SHAPES_ROW)
@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c5"])
def test_rowwise_rtn_small(name, shape):
    check_case(wl.make(name, *shape), tag=f"{name}-row")


@pytest.mark.parametrize("shape", SHAPES_COL)
@pytest.mark.parametrize("name", ["c1", "c3", "c4"])
def test_columnwise_rtn_small(name, shape):
    check_case(wl.make(name, *shape), layout=B.COLWISE, tag=f"{name}-col")


@pytest.mark.parametrize("shape", [(16, 16), (48, 176), (144, 272), (256, 384)])
def test_both_layouts_one_pass_small(shape):
    check_case(wl.make("c4", *shape), layout=B.BOTH, tag="c4-both")


@pytest.mark.parametrize("layout", [B.ROWWISE, B.COLWISE])
@pytest.mark.parametrize("select", [B.SEL_46_MSE, B.SEL_FORCE6, B.SEL_FORCE4, B.SEL_46_MAE,
                                    B.SEL_46_ABSMAX])
@pytest.mark.parametrize("rounding", [B.RTN, B.SR, B.SR_AFTER_RTN_SELECT])
@pytest.mark.parametrize("rht", [0, 1])
def test_option_matrix(layout, select, rounding, rht):
    check_case(wl.make("c5", 160, 304), layout=layout, rounding=rounding, select=select, rht=rht,
               tag="c5-matrix")


UNDERFLOW_KINDS = [k for k in wl.ADVERSARIAL_KINDS if k.startswith("sq_underflow")]


@pytest.mark.parametrize("kind", UNDERFLOW_KINDS)
@pytest.mark.parametrize("rounding,rht", [(B.RTN, 0), (B.SR, 0), (B.SR_AFTER_RTN_SELECT, 0),
                                          (B.RTN, 1), (B.SR, 1)])
def test_option_matrix_where_squared_errors_are_subnormal(kind, rounding, rht):
    """max|x| around 2^-58 ... 2^-72: the squared errors of Table 3 lines 6 / 12 are fp32
    subnormals (not all zero), so the 4-vs-6 decision rests on subnormal arithmetic and the
    kernel's error estimates are worthless there -- it has to evaluate the defined errors."""
    for dt in (torch.bfloat16, torch.float32):
        x = wl.adversarial(kind, 64, 256, dtype=dt)
        for layout in (B.ROWWISE, B.COLWISE):
            out = check_case(x, layout=layout, rounding=rounding, rht=rht, tag=f"{kind}-{dt}")
        if kind in ("sq_underflow_60", "sq_underflow_66", "sq_underflow_70", "sq_underflow_72"):
            sfx = "row" if layout == B.ROWWISE else "col"
            assert 0.05 < float(_np(out[f"choice_{sfx}"]).mean()) < 0.95


@pytest.mark.parametrize("rounding", [B.RTN, B.SR])
def test_both_layouts_with_sr(rounding):
    check_case(wl.make("c3", 144, 272), layout=B.BOTH, rounding=rounding, tag="c3-both")


@pytest.mark.parametrize("name", ["c1", "c2"])
def test_standard_tensor_scale_448(name):
    # with 448 in Eq. (1) the M=4 scale of the block that holds the maximum saturates
    check_case(wl.make(name, 64, 256), fp8_max=448.0, tag=f"{name}-448")
    check_case(wl.make(name, 64, 256), fp8_max=448.0, select=B.SEL_FORCE4, tag=f"{name}-448-f4")


@pytest.mark.parametrize("kind", wl.ADVERSARIAL_KINDS)
@pytest.mark.parametrize("layout", [B.ROWWISE, B.COLWISE, B.BOTH])
def test_adversarial_tensors(kind, layout):
    check_case(wl.adversarial(kind), layout=layout, tag=f"adv-{kind}")


def test_adversarial_with_sr_and_rht():
    for kind in wl.ADVERSARIAL_KINDS:
        check_case(wl.adversarial(kind), rounding=B.SR, rht=1, tag=f"adv-{kind}-sr-rht")


@pytest.mark.parametrize("layout", [B.ROWWISE, B.BOTH])
@pytest.mark.parametrize("rounding", [B.RTN, B.SR])
def test_decision_on_ties_and_near_ties(layout, rounding):
    """Blocks whose two candidates have equal or almost equal errors: the kernel decides
    most blocks from cheap error estimates and must fall back to the defined errors (or
    recognise an exact tie) on exactly these."""
    x = wl.adversarial("decision_stress", 1024, 2048)
    out = check_case(x, layout=layout, rounding=rounding, tag="decision-stress")
    frac4 = float(_np(out["choice_row"]).mean())
    assert 0.02 < frac4 < 0.9


@pytest.mark.parametrize("select", [B.SEL_46_MAE, B.SEL_46_ABSMAX])
@pytest.mark.parametrize("name,layout", [("c2", B.ROWWISE), ("c3", B.ROWWISE), ("c4", B.BOTH)])
def test_other_selection_rules(name, layout, select):
    # the mean-absolute-error and largest-absolute-error rules of Section 3.1 / Table 4
    x = wl.make(name, 1024, 2048)
    out = check_case(x, layout=layout, select=select, tag=f"{name}-sel{select}")
    frac4 = float(_np(out["choice_row"]).mean())
    assert 0.02 < frac4 < 0.9
    check_case(wl.adversarial("decision_stress", 256, 512), layout=layout, select=select,
               tag=f"stress-sel{select}")


@pytest.mark.parametrize("name,layout", [("c5", B.ROWWISE), ("c3", B.COLWISE), ("c4", B.BOTH)])
def test_sr_after_rtn_selection(name, layout):
    # Appendix A.3, second alternative: choose from round-to-nearest candidates, then SR
    x = wl.make(name, 512, 1024)
    check_case(x, layout=layout, rounding=B.SR_AFTER_RTN_SELECT, tag=f"{name}-sr-after-rtn")
    check_case(wl.adversarial("decision_stress", 256, 512), layout=layout,
               rounding=B.SR_AFTER_RTN_SELECT, tag="stress-sr-after-rtn")


@pytest.mark.parametrize("select", [B.SEL_46_MSE, B.SEL_FORCE6, B.SEL_FORCE4, B.SEL_46_MAE,
                                    B.SEL_46_ABSMAX])
@pytest.mark.parametrize("rounding", [B.RTN, B.SR, B.SR_AFTER_RTN_SELECT])
def test_block2d_matches_oracle(select, rounding):
    """One scale per 16x16 tile (the weight quantization named in Section 4.1)."""
    cases = [(wl.make("c2", 272, 400), "c2"), (wl.make("c4", 1024, 1024), "c4")]
    # tiles whose squared errors are fp32 subnormals, BF16 and FP32 input
    cases += [(wl.adversarial(k, 64, 256, dtype=dt), k) for k in UNDERFLOW_KINDS
              for dt in (torch.bfloat16, torch.float32)]
    for x, name in cases:
        _log(f"block2d case {name} {tuple(x.shape)} {x.dtype} select={select} rounding={rounding}")
        rows, cols = x.shape
        xb, xd = wl.host_array(x), x.cuda()
        alpha = B.nvfp4_46_tensor_scale(xd)
        a = float(alpha.item())
        kw = dict(rounding=rounding, select=select, sr_seed=SR_SEED)
        c_ref, s_ref, f_ref, d_ref = ref.quantize_2d(xb, a, **kw)
        out = B.nvfp4_46_quantize(xd, alpha, block2d=1, **kw)
        assert out["scales_row"].shape == (rows // 16, cols // 16)
        assert np.array_equal(_np(out["scales_row"]), s_ref)
        assert np.array_equal(_np(out["choice_row"]), f_ref)
        assert np.array_equal(_np(out["codes_row"]), c_ref)
        deq = B.nvfp4_46_dequantize(out["codes_row"], out["scales_row"], alpha, rows, cols,
                                    layout=B.BLOCK2D)
        assert np.array_equal(_bits(deq), d_ref)
        fq = B.nvfp4_46_fake_quant(xd, alpha, block2d=1, **kw)
        assert np.array_equal(_bits(fq), d_ref)


@pytest.mark.parametrize("layout", [B.BOTH, B.COLWISE])
@pytest.mark.parametrize("select,rounding", [(B.SEL_46_MSE, B.RTN), (B.SEL_46_MAE, B.SR),
                                             (B.SEL_FORCE6, B.SR_AFTER_RTN_SELECT)])
def test_block2d_packing_for_the_transposed_matrix(layout, select, rounding):
    """16x16 tiles are decided once; the columnwise outputs are the same codes and scales
    packed for W^T (oracle: plain re-indexing of its rowwise 2D outputs)."""
    for name, shape, dt in (("c2", (272, 400), torch.bfloat16), ("c4", (512, 1024), torch.float32)):
        x = wl.make(name, *shape, dtype=dt)
        rows, cols = shape
        xh, xd = wl.host_array(x), x.cuda()
        alpha = B.nvfp4_46_tensor_scale(xd)
        a = float(alpha.item())
        kw = dict(rounding=rounding, select=select, sr_seed=SR_SEED)
        c_ref, s_ref, f_ref, d_ref = ref.quantize_2d(xh, a, **kw)
        cc_ref, sc_ref, fc_ref = ref.repack_2d_columnwise(c_ref, s_ref, f_ref)
        out = B.nvfp4_46_quantize(xd, alpha, layout=layout, block2d=1, **kw)
        assert out["scales_col"].shape == (cols // 16, rows // 16)
        assert np.array_equal(_np(out["codes_col"]), cc_ref)
        assert np.array_equal(_np(out["scales_col"]), sc_ref)
        assert np.array_equal(_np(out["choice_col"]), fc_ref)
        if layout & B.ROWWISE:
            assert np.array_equal(_np(out["codes_row"]), c_ref)
            assert np.array_equal(_np(out["scales_row"]), s_ref)
        else:
            assert out["codes_row"] is None
        deq = B.nvfp4_46_dequantize(out["codes_col"], out["scales_col"], alpha, rows, cols,
                                    layout=B.BLOCK2D | B.COLWISE)
        assert np.array_equal(_bits(deq), d_ref)
        assert np.array_equal(ref.dequantize_2d_columnwise(cc_ref, sc_ref, a, rows, cols), d_ref)


def test_block2d_both_packings_past_one_round_of_the_grid():
    """4112 x 16400: 257 x 1025 tiles, so the last row and the last column of the kernel's work
    units (16 x 4 tiles) are ragged, and there are more units (4369) than workgroups in the
    grid (16 per compute unit), so workgroups take a second unit."""
    rows, cols = 4112, 16400
    x = wl.make("c2", rows, cols)
    xh, xd = wl.host_array(x), x.cuda()
    alpha = B.nvfp4_46_tensor_scale(xd)
    a = float(alpha.item())
    c_ref, s_ref, f_ref, _ = ref.quantize_2d(xh, a)
    cc_ref, sc_ref, fc_ref = ref.repack_2d_columnwise(c_ref, s_ref, f_ref)
    for layout in (B.BOTH, B.COLWISE, B.ROWWISE):
        _log(f"block2d at size: layout {layout}")
        out = B.nvfp4_46_quantize(xd, alpha, layout=layout, block2d=1)
        if layout & B.COLWISE:
            assert np.array_equal(_np(out["codes_col"]), cc_ref)
            assert np.array_equal(_np(out["scales_col"]), sc_ref)
            assert np.array_equal(_np(out["choice_col"]), fc_ref)
        if layout & B.ROWWISE:
            assert np.array_equal(_np(out["codes_row"]), c_ref)
            assert np.array_equal(_np(out["scales_row"]), s_ref)
            assert np.array_equal(_np(out["choice_row"]), f_ref)


@pytest.mark.parametrize("shape", [(16, 16), (16, 80), (272, 16), (32, 48), (64, 64)])
def test_block2d_smallest_shapes_in_every_packing(shape):
    """One tile, one row of tiles, one column of tiles, and less than one of the kernel's
    16 x 4-tile work units in either direction."""
    for layout in (B.ROWWISE, B.COLWISE, B.BOTH):
        check_case_2d(dict(name="c2", rows=shape[0], cols=shape[1], layout=layout, rounding=B.RTN,
                           select=B.SEL_46_MSE, f32=False), 9400, f"2d-small-{shape}-{layout}")


def _sweep_cases_2d(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        cases.append(dict(
            rows=int(rng.integers(1, 80)) * 16, cols=int(rng.integers(1, 120)) * 16,
            layout=int(rng.choice([B.ROWWISE, B.COLWISE, B.BOTH], p=[0.2, 0.2, 0.6])),
            rounding=int(rng.choice([B.RTN, B.SR, B.SR_AFTER_RTN_SELECT])),
            select=int(rng.choice([B.SEL_46_MSE, B.SEL_FORCE6, B.SEL_FORCE4, B.SEL_46_MAE,
                                   B.SEL_46_ABSMAX], p=[0.4, 0.1, 0.1, 0.2, 0.2])),
            name=str(rng.choice(["c1", "c2", "c3", "c5"])), f32=bool(rng.integers(0, 2))))
    return cases


def check_case_2d(c, seed, tag):
    _log(f"2d sweep {tag}: {c}")
    x = wl.make(c["name"], c["rows"], c["cols"], seed=seed,
                dtype=torch.float32 if c["f32"] else torch.bfloat16)
    xh, xd = wl.host_array(x), x.cuda()
    alpha = B.nvfp4_46_tensor_scale(xd)
    a = float(alpha.item())
    kw = dict(rounding=c["rounding"], select=c["select"], sr_seed=SR_SEED)
    c_ref, s_ref, f_ref, _ = ref.quantize_2d(xh, a, **kw)
    out = B.nvfp4_46_quantize(xd, alpha, layout=c["layout"], block2d=1, **kw)
    if c["layout"] & B.ROWWISE:
        assert np.array_equal(_np(out["codes_row"]), c_ref), tag
        assert np.array_equal(_np(out["scales_row"]), s_ref), tag
        assert np.array_equal(_np(out["choice_row"]), f_ref), tag
    if c["layout"] & B.COLWISE:
        cc_ref, sc_ref, fc_ref = ref.repack_2d_columnwise(c_ref, s_ref, f_ref)
        assert np.array_equal(_np(out["codes_col"]), cc_ref), tag
        assert np.array_equal(_np(out["scales_col"]), sc_ref), tag
        assert np.array_equal(_np(out["choice_col"]), fc_ref), tag


def test_seeded_sweep_of_block2d_shapes_and_options():
    """Thirty drawn combinations of tile-grid shape (ragged against the kernel's 16 x 4-tile work
    units), packing(s), rounding, rule and input type, each compared element by element."""
    for i, c in enumerate(_sweep_cases_2d(30, 4647)):
        check_case_2d(c, 9500 + i, f"2d-{i}")


@pytest.mark.parametrize("select", [B.SEL_46_MSE, B.SEL_46_MAE])
def test_blocks_within_a_few_steps_of_a_tie(select):
    """1x16 blocks (fp32 input) whose two candidates' errors cross within a few fp32 steps of one
    element (tests/_near_ties.py), fourteen steps around each crossing, under one alpha: the
    squared-error estimates cannot decide these, the kernels' defined-error path has to, in the
    stated order of additions (the absolute-error rule is always evaluated as defined, in the
    same order).  Rowwise, and the same blocks laid along columns."""
    from tests._near_ties import BLOCK_STEPS, block_crossings
    from tests.test_oracle_order_transcriptions import _tree_of_halves
    alpha = float(np.float32(1.0) / np.float32(1536.0))
    blocks = []
    metric = None if select == B.SEL_46_MSE else ref.SEL_46_MAE
    for v, i, first, _, _ in block_crossings(800, 4696, _tree_of_halves, alpha, metric):
        for step in BLOCK_STEPS:
            w = v.copy()
            w[i] = np.uint32(first + step).view(np.float32)
            blocks.append(w)
    n = len(blocks) // 256 * 256
    assert n >= 2048, n
    x = np.stack(blocks[:n]).reshape(n // 16, 256)            # 16 blocks per row
    _log(f"near-tie blocks: {n} blocks, tensor {x.shape}")
    ad = torch.tensor([alpha], dtype=torch.float32, device="cuda")
    c_ref, s_ref, f_ref = ref.quantize(x, alpha, select=select)
    assert 0.25 < f_ref.mean() < 0.75
    out = B.nvfp4_46_quantize(torch.from_numpy(x).cuda(), ad, select=select)
    assert np.array_equal(_np(out["choice_row"]), f_ref)
    assert np.array_equal(_np(out["scales_row"]), s_ref)
    assert np.array_equal(_np(out["codes_row"]), c_ref)
    # the same blocks along columns: x^T, quantized columnwise and in both orientations at once
    xt = np.ascontiguousarray(x.T)                            # [256][n/16]: rows % 16 == 0
    c_ref, s_ref, f_ref = ref.quantize(xt, alpha, layout=ref.COLWISE, select=select)
    assert 0.25 < f_ref.mean() < 0.75
    for layout in (B.COLWISE, B.BOTH):
        out = B.nvfp4_46_quantize(torch.from_numpy(xt).cuda(), ad, layout=layout, select=select)
        assert np.array_equal(_np(out["choice_col"]), f_ref)
        assert np.array_equal(_np(out["scales_col"]), s_ref)
        assert np.array_equal(_np(out["codes_col"]), c_ref)


def test_stochastically_rounded_blocks_within_a_step_of_a_tie():
    """The same with stochastic rounding: every block is built for its own place in the tensor
    (its uniforms are those of its elements' indices) so that its two stochastically rounded
    candidates' errors cross between two adjacent fp32 values of one element; the element sits
    on one side or the other of the crossing, alternating."""
    from tests._near_ties import block_crossings
    from tests.test_oracle_order_transcriptions import _tree_of_halves
    alpha = float(np.float32(1.0) / np.float32(1536.0))
    cols = 256

    def uniforms(k):                      # block k -> row k // 16, columns 16 (k % 16) ...
        g0 = (k // 16) * cols + 16 * (k % 16)
        return np.array([ref.sr_uniform(SR_SEED, g0 + j) for j in range(16)], np.float32)

    blocks = []
    for v, i, first, _, _ in block_crossings(6000, 4697, _tree_of_halves, alpha, None, ref.SR, uniforms,
                                             samples=24, elements=4):
        w = v.copy()
        w[i] = np.uint32(first + (-1, 0, 1, 2)[len(blocks) % 4]).view(np.float32)
        blocks.append(w)
        if len(blocks) == 512:
            break
    assert len(blocks) == 512
    x = np.stack(blocks).reshape(32, cols)
    c_ref, s_ref, f_ref = ref.quantize(x, alpha, rounding=ref.SR, sr_seed=SR_SEED)
    assert 0.25 < f_ref.mean() < 0.75
    ad = torch.tensor([alpha], dtype=torch.float32, device="cuda")
    out = B.nvfp4_46_quantize(torch.from_numpy(x).cuda(), ad, rounding=B.SR, sr_seed=SR_SEED)
    assert np.array_equal(_np(out["choice_row"]), f_ref)
    assert np.array_equal(_np(out["scales_row"]), s_ref)
    assert np.array_equal(_np(out["codes_row"]), c_ref)


def test_block2d_tiles_within_a_few_steps_of_a_tie():
    """Tiles whose two candidates' errors cross between two adjacent fp32 values of one element
    (tests/_near_ties.py), eighteen steps around each crossing, one tile each, under one common
    alpha: the estimates cannot decide these, so the kernel's defined-error path and the order
    in which sixteen lanes add their row errors decide them; choices must equal the oracle's."""
    from tests._near_ties import STEPS, crossings
    from tests.test_oracle_order_transcriptions import _tree_of_halves
    alpha = float(np.float32(1.0) / np.float32(1536.0))
    tiles = []
    for t, r, c, first, _, _, _ in crossings(400, 4694, _tree_of_halves, alpha=alpha):
        for step in STEPS:
            tile = t.copy()
            tile[r, c] = np.uint32(first + step).view(np.float32)
            tiles.append(tile)
    n = len(tiles) // 16 * 16
    assert n >= 256, n
    x = np.block([[tiles[16 * i + j] for j in range(16)] for i in range(n // 16)])   # [n][256]
    _log(f"near-tie tiles: {n} tiles, tensor {x.shape}")
    c_ref, s_ref, f_ref, _ = ref.quantize_2d(x, alpha)
    assert 0.2 < f_ref.mean() < 0.8                       # they do go both ways
    xd = torch.from_numpy(x).cuda()
    ad = torch.tensor([alpha], dtype=torch.float32, device="cuda")
    for layout in (B.ROWWISE, B.BOTH):
        out = B.nvfp4_46_quantize(xd, ad, layout=layout, block2d=1)
        assert np.array_equal(_np(out["choice_row"]), f_ref)
        assert np.array_equal(_np(out["scales_row"]), s_ref)
        assert np.array_equal(_np(out["codes_row"]), c_ref)
    cc_ref, sc_ref, fc_ref = ref.repack_2d_columnwise(c_ref, s_ref, f_ref)
    assert np.array_equal(_np(out["choice_col"]), fc_ref)
    assert np.array_equal(_np(out["codes_col"]), cc_ref)


def test_block2d_transpose_consistency_on_gpu():
    # under a fixed scale rule, quantizing W^T with 16x16 tiles is the transpose of quantizing W
    x = wl.make("c2", 512, 768)
    xd, xtd = x.cuda(), x.t().contiguous().cuda()
    alpha = B.nvfp4_46_tensor_scale(xd)
    d = B.nvfp4_46_fake_quant(xd, alpha, select=B.SEL_FORCE6, block2d=1)
    dt = B.nvfp4_46_fake_quant(xtd, alpha, select=B.SEL_FORCE6, block2d=1)
    assert torch.equal(dt, d.t().contiguous())


# ------------------------------------------------------------------ fp32 input (FP32 master weights)

@pytest.mark.parametrize("shape", [(16, 16), (144, 272), (257, 48), (1000, 4112)])
def test_fp32_input_rowwise(shape):
    check_case(wl.make("c2", *shape, dtype=torch.float32), tag="c2-f32-row")


@pytest.mark.parametrize("shape", [(16, 8), (144, 264), (272, 136), (1008, 4104)])
def test_fp32_input_columnwise(shape):
    check_case(wl.make("c2", *shape, dtype=torch.float32), layout=B.COLWISE, tag="c2-f32-col")


@pytest.mark.parametrize("shape", [(48, 176), (256, 384), (1008, 2064)])
def test_fp32_input_both_layouts(shape):
    check_case(wl.make("c4", *shape, dtype=torch.float32), layout=B.BOTH, tag="c4-f32-both")


@pytest.mark.parametrize("layout", [B.ROWWISE, B.COLWISE])
@pytest.mark.parametrize("select", [B.SEL_46_MSE, B.SEL_FORCE4, B.SEL_46_MAE, B.SEL_46_ABSMAX])
@pytest.mark.parametrize("rounding,rht", [(B.RTN, 0), (B.SR, 1), (B.SR_AFTER_RTN_SELECT, 0),
                                          (B.RTN, 1)])
def test_fp32_input_option_matrix(layout, select, rounding, rht):
    check_case(wl.make("c5", 160, 304, dtype=torch.float32), layout=layout, rounding=rounding,
               select=select, rht=rht, tag="c5-f32-matrix")


@pytest.mark.parametrize("kind", ["zeros", "neg_zeros", "one_hot", "tiny", "wide_range", "ties",
                                  "bf16_small", "bf16_large"] + UNDERFLOW_KINDS)
def test_fp32_input_adversarial(kind):
    check_case(wl.adversarial(kind, dtype=torch.float32), layout=B.BOTH, tag=f"adv-f32-{kind}")


def test_fp32_input_decision_stress():
    x = wl.adversarial("decision_stress", 1024, 2048, dtype=torch.float32)
    out = check_case(x, layout=B.BOTH, tag="decision-stress-f32")
    assert 0.02 < float(_np(out["choice_row"]).mean()) < 0.9


@pytest.mark.parametrize("select", [B.SEL_FORCE6, B.SEL_46_MSE])
def test_stochastic_rounding_at_its_thresholds_end_to_end(select):
    """FP32 values placed within a few 2^-25 of the threshold their own uniform sets (the uniform
    of an element is known from the seed and its index): the cases in which the conversion
    instruction alone would round differently from the stated rule, so the kernel's margin test
    and its software path decide most blocks here.  Every block's maximum is 6 and alpha is 1,
    so under the scale-to-6 candidate the scaled value is the input itself."""
    rows, cols = 64, 256
    rng = np.random.default_rng(77)
    k = np.array([round(ref.sr_uniform(SR_SEED, g) * 2.0 ** 24) for g in range(rows * cols)],
                 np.int64).reshape(rows, cols)
    d = rng.integers(-3, 4, (rows, cols))
    half = rng.random((rows, cols)) < 0.5                   # lower grid point 0.5 instead of 0
    n = np.clip(k + d, 0, (1 << 24) - 2)
    n = np.where(half, n & ~1, n)                           # 2^24 + n must fit 24 bits: even n
    mag = np.where(half, 0.5, 0.0) + n.astype(np.float64) * 2.0 ** -25
    x = (mag * rng.choice([-1.0, 1.0], (rows, cols))).astype(np.float32)
    assert np.array_equal(np.abs(x).astype(np.float64), mag)   # exactly representable
    x[:, ::16] = 6.0
    xt = torch.from_numpy(x)
    # how many of these the instruction alone gets wrong (diagnostic, through the debug entry)
    words = torch.from_numpy(((k << 8) | 0x33).astype(np.uint32).view(np.int32).reshape(-1)).cuda()
    got, fast = B.nvfp4_46_debug_e2m1_sr(xt.reshape(-1).cuda(), words)
    wrong = ((fast & 0x0F) != got).float().mean().item()
    flagged = ((fast & 0x80) != 0).float().mean().item()
    _log(f"instruction alone differs on {wrong:.3f} of the elements, margin test fires on {flagged:.3f}")
    assert wrong > 0.05 and flagged > 0.5
    check_case(xt, rounding=B.SR, select=select, alpha_value=1.0, tag="sr-thresholds")
    check_case(xt, layout=B.COLWISE, rounding=B.SR, select=select, alpha_value=1.0, tag="sr-thresholds-col")


def test_fp32_input_sees_the_low_mantissa_bits():
    """The fp32 path must not round x to BF16 on the way in: its result differs from that of
    the BF16-rounded tensor, and equals it when the values are BF16 values to begin with."""
    xf = wl.make("c2", 256, 512, dtype=torch.float32)
    xr = xf.to(torch.bfloat16)
    alpha = B.nvfp4_46_tensor_scale(xf.cuda())
    o32 = B.nvfp4_46_quantize(xf.cuda(), alpha)
    o16 = B.nvfp4_46_quantize(xr.cuda(), alpha)
    assert not torch.equal(o32["codes_row"], o16["codes_row"])
    o16f = B.nvfp4_46_quantize(xr.float().cuda(), alpha)
    for k in ("codes_row", "scales_row", "choice_row"):
        assert torch.equal(o16f[k], o16[k])


@pytest.mark.parametrize("select", [B.SEL_46_MSE, B.SEL_46_MAE])
@pytest.mark.parametrize("rounding", [B.RTN, B.SR])
def test_fp32_input_block2d(select, rounding):
    x = wl.make("c2", 272, 400, dtype=torch.float32)
    rows, cols = x.shape
    xd = x.cuda()
    alpha = B.nvfp4_46_tensor_scale(xd)
    a = float(alpha.item())
    assert _alpha_bits(a) == _alpha_bits(ref.tensor_scale(x.numpy()))
    kw = dict(rounding=rounding, select=select, sr_seed=SR_SEED)
    c_ref, s_ref, f_ref, d_ref = ref.quantize_2d(x.numpy(), a, **kw)
    out = B.nvfp4_46_quantize(xd, alpha, block2d=1, **kw)
    assert np.array_equal(_np(out["scales_row"]), s_ref)
    assert np.array_equal(_np(out["choice_row"]), f_ref)
    assert np.array_equal(_np(out["codes_row"]), c_ref)
    assert np.array_equal(_bits(B.nvfp4_46_fake_quant(xd, alpha, block2d=1, **kw)), d_ref)


def test_caller_supplied_alpha_replays_table3():
    # Table 3's blocks with the tensor scale written as 1: [10,20,30,40] -> 4, [15,30,120,180] -> 6
    x = torch.zeros((16, 32), dtype=torch.float32)
    x[0, 0:4] = torch.tensor([10.0, 20.0, 30.0, 40.0])
    x[0, 16:20] = torch.tensor([15.0, 30.0, 120.0, 180.0])
    out = check_case(x.to(torch.bfloat16), alpha_value=1.0, tag="table3")
    assert _np(out["choice_row"])[0].tolist() == [1, 0]
    assert _np(out["scales_row"])[0].tolist() == [ref.e4m3_encode(10.0), ref.e4m3_encode(30.0)]
    assert _np(out["codes_row"])[0, :2].tolist() == [0x42, 0x65]       # [1,2,3,4]
    assert _np(out["codes_row"])[0, 8:10].tolist() == [0x21, 0x76]     # [.5,1,4,6]


def test_exact_error_ties_keep_six():
    # every block is exactly representable under both scalings -> E4 == E6 == 0 -> 6
    x = wl.adversarial("grid_exact")
    out = check_case(x, alpha_value=0.25 / 8, tag="ties")
    assert int(_np(out["choice_row"]).sum()) == 0


def test_optional_choice_and_preallocated_outputs():
    x = wl.make("c1", 64, 256)
    xd = x.cuda()
    alpha = B.nvfp4_46_tensor_scale(xd)
    full = B.nvfp4_46_quantize(xd, alpha, layout=B.BOTH)
    lean = B.nvfp4_46_quantize(xd, alpha, layout=B.BOTH, want_choice=False)
    assert lean["choice_row"] is None and lean["choice_col"] is None
    for k in ("codes_row", "scales_row", "codes_col", "scales_col"):
        assert torch.equal(full[k], lean[k])
    again = B.nvfp4_46_quantize(xd, alpha, layout=B.BOTH, out=full)      # in place, same result
    for k in ("codes_row", "scales_row", "codes_col", "scales_col"):
        assert torch.equal(again[k], lean[k])


def test_runs_on_a_side_stream_and_is_deterministic():
    x = wl.make("c3", 512, 1024)
    xd = x.cuda()
    s = torch.cuda.Stream()
    base = B.nvfp4_46_quantize(xd, B.nvfp4_46_tensor_scale(xd))
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        alpha = B.nvfp4_46_tensor_scale(xd, stream=s)
        outs = [B.nvfp4_46_quantize(xd, alpha, stream=s) for _ in range(3)]
    s.synchronize()
    for o in outs:
        for k in ("codes_row", "scales_row", "choice_row"):
            assert torch.equal(o[k], base[k])


def test_step_can_be_captured_in_a_graph_and_replayed():
    """tensor_scale -> quantize -> dequantize recorded into a HIP graph (the library only
    launches kernels on the stream it is given: no allocation, no memset, no sync) and
    replayed with eager work in between; every replay must equal the eager result."""
    x1 = wl.make("c2", 512, 1024)
    x2 = wl.make("c3", 512, 1024)
    xd = x1.cuda()
    rows, cols = xd.shape
    alpha = torch.empty(1, dtype=torch.float32, device="cuda")
    out = B.alloc_outputs(rows, cols, B.BOTH, "cuda")
    deq = torch.empty_like(xd)
    p = B.make_params(rows, cols, layout=B.BOTH)

    def step(stream):
        assert B.tensor_scale_raw(xd, p, alpha, stream) == 0
        assert B.quantize_raw(xd, p, alpha, out["codes_row"], out["scales_row"], out["codes_col"],
                              out["scales_col"], out["choice_row"], out["choice_col"], stream) == 0
        assert B.dequantize_raw(out["codes_row"], out["scales_row"], alpha, rows, cols, B.ROWWISE,
                                deq, stream) == 0

    def snapshot():
        torch.cuda.synchronize()
        return [alpha.clone(), deq.clone()] + [out[k].clone() for k in sorted(out)]

    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        step(s)                       # warm-up outside the capture
    s.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        step(torch.cuda.current_stream())
    for src in (x1, x2, x1, x2):
        xd.copy_(src.cuda())
        step(torch.cuda.current_stream())
        want = snapshot()
        for t in [alpha, deq] + [out[k] for k in out]:
            t.zero_()                 # eager work between the replays
        g.replay()
        got = snapshot()
        assert all(torch.equal(a, b) for a, b in zip(got, want))


def test_gpu_error_paths_enqueue_nothing():
    x = wl.make("c1", 32, 64).cuda()
    alpha = torch.ones(1, dtype=torch.float32, device="cuda")
    out = B.alloc_outputs(32, 64, B.ROWWISE, x.device)
    out["codes_row"].fill_(0xAB)
    p = B.make_params(32, 64, select=7)
    rc = B.quantize_raw(x, p, alpha, out["codes_row"], out["scales_row"], None, None, None, None)
    torch.cuda.synchronize()
    assert rc == 4 and bool((out["codes_row"] == 0xAB).all())
    with pytest.raises(B.Nvfp4Error):
        B.nvfp4_46_fake_quant(x, alpha, layout=B.BOTH)


# ------------------------------------------------------------------ the five workloads, full size

def test_workload_c1_full():
    check_case(wl.make("c1"), tag="c1-full")


def test_workload_c2_full_rowwise_rtn_and_mse():
    x = wl.make("c2")
    out = check_case(x, tag="c2-full")
    frac4 = float(_np(out["choice_row"]).mean())
    _log(f"c2: fraction of blocks scaled to 4 = {frac4:.4f}")
    assert 0.05 < frac4 < 0.7
    # 4/6 never has a larger tensor MSE than scale-to-6-only at the same alpha
    xd = x.cuda()
    alpha = B.nvfp4_46_tensor_scale(xd)
    xf = xd.double()
    mse46 = float(((B.nvfp4_46_fake_quant(xd, alpha).double() - xf) ** 2).mean())
    mse6 = float(((B.nvfp4_46_fake_quant(xd, alpha, select=B.SEL_FORCE6).double() - xf) ** 2).mean())
    _log(f"c2: MSE 4/6 = {mse46:.6e}, MSE scale-to-6 = {mse6:.6e}, ratio {mse46 / mse6:.4f}")
    assert mse46 <= mse6


def test_workload_c2_full_fp32_weights_both_layouts():
    # the weight matrix of Fig. 3 as stored (FP32), both operand orientations from one read
    check_case(wl.make("c2", dtype=torch.float32), layout=B.BOTH, tag="c2-f32-full")


def test_workload_c3_full_fake_quant():
    check_case(wl.make("c3"), tag="c3-full")


def test_workload_c4_full_both_layouts():
    check_case(wl.make("c4"), layout=B.BOTH, tag="c4-full")


def test_workload_c5_full_rht_sr():
    check_case(wl.make("c5"), rounding=B.SR, rht=1, tag="c5-full")


@pytest.mark.parametrize("dtype,rows,cols", [(torch.bfloat16, 8192, 8192), (torch.float32, 4096, 6152),
                                             (torch.bfloat16, 16, 8), (torch.float32, 48, 8)])
def test_tensor_scale_of_hadamard_transformed_columns_at_size(dtype, rows, cols):
    """The columnwise maximum after the transform (many rounds of the grid, a ragged last
    round, and the smallest legal tensors) equals the oracle's, bit for bit."""
    x = wl.make("c5", rows, cols, dtype=dtype)
    a_ref = ref.tensor_scale(wl.host_array(x), layout=ref.COLWISE, rht=1, rht_seed=RHT_SEED)
    a_gpu = B.nvfp4_46_tensor_scale(x.cuda(), layout=B.COLWISE, rht=1, rht_seed=RHT_SEED)
    assert _alpha_bits(a_gpu.item()) == _alpha_bits(a_ref)
    if cols % 16 == 0:          # the rowwise pass over the same tensor
        a_ref = ref.tensor_scale(wl.host_array(x), rht=1, rht_seed=RHT_SEED)
        a_gpu = B.nvfp4_46_tensor_scale(x.cuda(), rht=1, rht_seed=RHT_SEED)
        assert _alpha_bits(a_gpu.item()) == _alpha_bits(a_ref)


# ------------------------------------------------------------------ seeded sweep over shapes and options

def _sweep_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < n:
        layout = int(rng.choice([B.ROWWISE, B.COLWISE, B.BOTH]))
        rht = int(rng.integers(0, 2)) if layout != B.BOTH else 0
        rows = int(rng.integers(1, 40)) * 16 if layout != B.ROWWISE else int(rng.integers(1, 400))
        cols = int(rng.integers(1, 70)) * 16 if layout & B.ROWWISE else int(rng.integers(1, 140)) * 8
        cases.append(dict(
            rows=rows, cols=cols, layout=layout, rht=rht,
            rounding=int(rng.choice([B.RTN, B.SR, B.SR_AFTER_RTN_SELECT])),
            select=int(rng.choice([B.SEL_46_MSE, B.SEL_FORCE6, B.SEL_FORCE4, B.SEL_46_MAE,
                                   B.SEL_46_ABSMAX], p=[0.4, 0.1, 0.1, 0.2, 0.2])),
            name=str(rng.choice(["c1", "c2", "c3", "c5"])),
            f32=bool(rng.integers(0, 2)), fp8_max=float(rng.choice([256.0, 448.0], p=[0.8, 0.2]))))
    return cases


@pytest.mark.parametrize("chunk", range(6))
def test_seeded_sweep_of_shapes_and_options(chunk):
    """Sixty drawn combinations of shape, layout, rounding, rule, transform, input type and
    Eq. (1) constant, ten per test, each compared element by element."""
    for i, c in enumerate(_sweep_cases(60, 4646)[10 * chunk:10 * chunk + 10]):
        x = wl.make(c["name"], c["rows"], c["cols"], seed=9000 + 10 * chunk + i,
                    dtype=torch.float32 if c["f32"] else torch.bfloat16)
        check_case(x, layout=c["layout"], rounding=c["rounding"], select=c["select"], rht=c["rht"],
                   fp8_max=c["fp8_max"], tag=f"sweep-{chunk}-{i}-{c['name']}-f32={c['f32']}")


# ------------------------------------------------------------------ beyond 2^32 bytes

def test_tensor_larger_than_four_gibibytes():
    """65,552 x 40,960 BF16 = 2.69 G elements, 5.4 GB: element indices pass 2^31 and byte offsets
    2^32 inside one call.  The tensor is drawn on the GPU (seeded N(0,1), plus one planted
    maximum near the end); the oracle computes the tensor scale over all of it and quantizes
    32-row slices at the start, around the 2^31-byte, 2^32-byte and 2^31-element marks and at
    the end, each compared with the same slice of the GPU's outputs: rowwise + columnwise in
    one pass, and rowwise with the Hadamard transform and stochastic rounding (whose random
    numbers are keyed by the 64-bit element index)."""
    rows, cols = 65552, 40960
    g = torch.Generator(device="cuda")
    g.manual_seed(4650)
    x = torch.empty((rows, cols), dtype=torch.bfloat16, device="cuda")
    for r0 in range(0, rows, 8192):                          # drawn in pieces to bound temporaries
        n = min(8192, rows - r0)
        x[r0:r0 + n] = torch.randn((n, cols), generator=g, device="cuda", dtype=torch.float32)
    x[rows - 3, cols - 5] = 9.0
    marks = [0, (2 ** 30 // cols) // 16 * 16, (2 ** 31 // cols) // 16 * 16 - 16, rows - 32]
    marks.insert(2, (2 ** 31 // cols) // 16 * 16 // 2 * 2)   # 2^32 bytes = 2^31 elements
    marks = sorted(set(marks))
    _log(f"big tensor: slices at rows {marks}")

    alpha = B.nvfp4_46_tensor_scale(x)
    assert _alpha_bits(alpha.item()) == _alpha_bits(np.float32(9.0) / np.float32(1536.0))
    a = float(alpha.item())
    slices = {r0: x[r0:r0 + 32].cpu().view(torch.int16).numpy().view(np.uint16).copy() for r0 in marks}

    out = B.nvfp4_46_quantize(x, alpha, layout=B.BOTH)
    torch.cuda.synchronize()
    for r0, xb in slices.items():
        c, s, f, _ = ref.quantize_rows(xb, r0, a, layout=ref.ROWWISE)
        assert np.array_equal(_np(out["codes_row"][r0:r0 + 32]), c), r0
        assert np.array_equal(_np(out["scales_row"][r0:r0 + 32]), s), r0
        assert np.array_equal(_np(out["choice_row"][r0:r0 + 32]), f), r0
        c, s, f, _ = ref.quantize_rows(xb, r0, a, layout=ref.COLWISE)
        assert np.array_equal(_np(out["codes_col"][:, r0 // 2:r0 // 2 + 16]), c), r0
        assert np.array_equal(_np(out["scales_col"][:, r0 // 16:r0 // 16 + 2]), s), r0
    del out
    torch.cuda.empty_cache()

    kw = dict(rounding=B.SR, rht=1, sr_seed=SR_SEED, rht_seed=RHT_SEED)
    a_t = B.nvfp4_46_tensor_scale(x, rht=1, rht_seed=RHT_SEED)
    out = B.nvfp4_46_quantize(x, a_t, want_choice=False, **kw)
    fq = B.nvfp4_46_fake_quant(x, a_t, **kw)
    torch.cuda.synchronize()
    for r0, xb in slices.items():
        c, s, _, d = ref.quantize_rows(xb, r0, float(a_t.item()), **kw)
        assert np.array_equal(_np(out["codes_row"][r0:r0 + 32]), c), r0
        assert np.array_equal(_np(out["scales_row"][r0:r0 + 32]), s), r0
        assert np.array_equal(_bits(fq[r0:r0 + 32]), d), r0


def test_tensor_scale_workspace_is_left_zeroed_and_full_size_matches():
    ws = B.new_workspace()
    for name in ("c2", "c5"):
        x = wl.make(name, 4096, 8192)
        xb, xd = wl.bf16_bits(x), x.cuda()
        for kw in (dict(), dict(rht=1, rht_seed=RHT_SEED), dict(rht=1, rht_seed=RHT_SEED, layout=B.COLWISE)):
            a_ref = ref.tensor_scale(xb, **{k: (ref.COLWISE if v == B.COLWISE else v) for k, v in kw.items()})
            for _ in range(3):
                a = B.nvfp4_46_tensor_scale_ws(xd, ws, **kw)
                assert _alpha_bits(a.item()) == _alpha_bits(a_ref), (name, kw)
                assert int(ws.cpu().sum()) == 0
    # an all-zero tensor: alpha = 1
    z = torch.zeros((64, 256), dtype=torch.bfloat16, device="cuda")
    assert B.nvfp4_46_tensor_scale_ws(z, ws).item() == 1.0
