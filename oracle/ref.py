"""ctypes binding of the CPU oracle (``oracle/nvfp4_46_ref.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by
the benchmark's CPU-baseline leg.  Nothing in the product package imports it.

The oracle is compiled with gcc into ``oracle/libnvfp4_46_ref.so`` by
:func:`build`; :func:`lib` loads it (building it first if it is absent).
All arrays are numpy arrays in host memory.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "nvfp4_46_ref.c"
_SO = _HERE / "libnvfp4_46_ref.so"

RTN, SR, SR_AFTER_RTN_SELECT = 0, 1, 2
SEL_46_MSE, SEL_FORCE6, SEL_FORCE4, SEL_46_MAE, SEL_46_ABSMAX = 0, 1, 2, 3, 4
ROWWISE, COLWISE = 1, 2

# no FMA contraction, no fast-math, default (round-to-nearest) mode, SSE2 fp32
CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
          "-fno-fast-math", "-fno-unsafe-math-optimizations", "-Wall", "-Wextra"]


def build(force: bool = True) -> Path:
    if _SO.exists() and not force and _SO.stat().st_mtime >= _SRC.stat().st_mtime:
        return _SO
    tmp = _SO.with_suffix(f".tmp{os.getpid()}.so")
    subprocess.run(["gcc", *CFLAGS, str(_SRC), "-o", str(tmp), "-lm"], check=True)
    os.replace(tmp, _SO)
    return _SO


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        # NVFP4_46_REF_LIB names another build of the oracle to load instead (the mutation
        # test points the pin tests at deliberately broken copies this way)
        other = os.environ.get("NVFP4_46_REF_LIB")
        if not other:
            build(force=False)
        L = C.CDLL(other or str(_SO))
        u8p, u16p, f32p, u32p = (C.POINTER(C.c_uint8), C.POINTER(C.c_uint16),
                                 C.POINTER(C.c_float), C.POINTER(C.c_uint32))
        i64, u64, i32, f32 = C.c_int64, C.c_uint64, C.c_int, C.c_float
        L.ref_bf16_to_f32.restype, L.ref_bf16_to_f32.argtypes = f32, [C.c_uint16]
        L.ref_f32_to_bf16.restype, L.ref_f32_to_bf16.argtypes = C.c_uint16, [f32]
        L.ref_e2m1_decode.restype, L.ref_e2m1_decode.argtypes = f32, [C.c_uint8]
        L.ref_e2m1_rtn.restype, L.ref_e2m1_rtn.argtypes = C.c_uint8, [f32]
        L.ref_e2m1_sr.restype, L.ref_e2m1_sr.argtypes = C.c_uint8, [f32, f32]
        L.ref_e4m3_decode.restype, L.ref_e4m3_decode.argtypes = f32, [C.c_uint8]
        L.ref_e4m3_encode.restype, L.ref_e4m3_encode.argtypes = C.c_uint8, [f32]
        L.ref_philox4x32_10.restype, L.ref_philox4x32_10.argtypes = None, [u32p, u32p, u32p]
        L.ref_sr_uniform.restype, L.ref_sr_uniform.argtypes = f32, [u64, u64]
        L.ref_rht_sign_word.restype, L.ref_rht_sign_word.argtypes = C.c_uint32, [u64, u64]
        L.ref_rht16.restype, L.ref_rht16.argtypes = None, [f32p, C.c_uint32]
        L.ref_block_scale.restype, L.ref_block_scale.argtypes = C.c_uint8, [f32, f32, f32]
        L.ref_block_with_scale.restype = f32
        L.ref_block_with_scale.argtypes = [f32p, f32, C.c_uint8, i32, f32p, u8p, f32p]
        L.ref_quantize_block.restype = None
        L.ref_quantize_block.argtypes = [f32p, f32, i32, i32, f32p, u8p, f32p, u8p, u8p, f32p]
        L.nvfp4_46_ref_tensor_scale.restype = i32
        L.nvfp4_46_ref_tensor_scale.argtypes = [u16p, i64, i64, i32, i32, u64, f32, f32p]
        L.nvfp4_46_ref_quantize.restype = i32
        L.nvfp4_46_ref_quantize.argtypes = [u16p, i64, i64, i32, i32, i32, i32, u64, u64, f32,
                                            u8p, u8p, u8p, u16p]
        L.nvfp4_46_ref_tensor_scale_f32.restype = i32
        L.nvfp4_46_ref_tensor_scale_f32.argtypes = [f32p, i64, i64, i32, i32, u64, f32, f32p]
        L.nvfp4_46_ref_quantize_f32.restype = i32
        L.nvfp4_46_ref_quantize_f32.argtypes = [f32p, i64, i64, i32, i32, i32, i32, u64, u64, f32,
                                                u8p, u8p, u8p, u16p]
        L.nvfp4_46_ref_quantize_2d_f32.restype = i32
        L.nvfp4_46_ref_quantize_2d_f32.argtypes = [f32p, i64, i64, i32, i32, u64, f32, u8p, u8p,
                                                   u8p, u16p]
        L.nvfp4_46_ref_quantize_rows.restype = i32
        L.nvfp4_46_ref_quantize_rows.argtypes = [u16p, i64, i64, i64, i32, i32, i32, i32, u64, u64,
                                                 f32, u8p, u8p, u8p, u16p]
        L.nvfp4_46_ref_dequantize.restype = i32
        L.nvfp4_46_ref_dequantize.argtypes = [u8p, u8p, f32, i64, i64, i32, u16p]
        L.nvfp4_46_ref_fake_quant.restype = i32
        L.nvfp4_46_ref_fake_quant.argtypes = [u16p, i64, i64, i32, i32, i32, i32, u64, u64, f32,
                                              u16p]
        L.nvfp4_46_ref_block_errors_sel.restype = i32
        L.nvfp4_46_ref_block_errors_sel.argtypes = [u16p, i64, i64, i32, i32, i32, i32, u64, u64,
                                                    f32, f32p, f32p]
        L.ref_block_abs_metric.restype = f32
        L.ref_block_abs_metric.argtypes = [f32p, f32p, i32]
        L.nvfp4_46_ref_quantize_2d.restype = i32
        L.nvfp4_46_ref_quantize_2d.argtypes = [u16p, i64, i64, i32, i32, u64, f32, u8p, u8p, u8p,
                                               u16p]
        L.nvfp4_46_ref_repack_2d_columnwise.restype = i32
        L.nvfp4_46_ref_repack_2d_columnwise.argtypes = [u8p, u8p, u8p, i64, i64, u8p, u8p, u8p]
        L.nvfp4_46_ref_dequantize_2d_columnwise.restype = i32
        L.nvfp4_46_ref_dequantize_2d_columnwise.argtypes = [u8p, u8p, f32, i64, i64, u16p]
        L.nvfp4_46_ref_dequantize_2d.restype = i32
        L.nvfp4_46_ref_dequantize_2d.argtypes = [u8p, u8p, f32, i64, i64, u16p]
        f64p = C.POINTER(C.c_double)
        L.nvfp4_46_ref_gemm.restype = i32
        L.nvfp4_46_ref_gemm.argtypes = [u8p, u8p, f32, u8p, u8p, f32, i64, i64, i64, i32, i32,
                                        f64p, f64p]
        L.ref_e2m1_rtn_bits_range.restype = None
        L.ref_e2m1_rtn_bits_range.argtypes = [C.c_uint32, i64, u8p]
        L.ref_e2m1_sr_bits_range.restype = None
        L.ref_e2m1_sr_bits_range.argtypes = [C.c_uint32, i64, C.c_float, u8p]
        L.ref_e2m1_sr_n.restype = None
        L.ref_e2m1_sr_n.argtypes = [f32p, f32p, i64, u8p]
        L.ref_e4m3_encode_bits_range.restype = None
        L.ref_e4m3_encode_bits_range.argtypes = [C.c_uint32, i64, u8p]
        _lib = L
    return _lib


def _p(a: np.ndarray | None, ctype):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(ctype))


def _check_x(x_bits: np.ndarray):
    """The input tensor: uint16 = BF16 bit patterns, float32 = fp32 values."""
    assert x_bits.dtype in (np.uint16, np.float32) and x_bits.ndim == 2
    assert x_bits.flags["C_CONTIGUOUS"]
    return x_bits.shape


def _x(x: np.ndarray, name: str):
    """(C function, pointer) for the input's element type."""
    if x.dtype == np.float32:
        return getattr(lib(), name + "_f32"), _p(x, C.c_float)
    return getattr(lib(), name), _p(x, C.c_uint16)


def _out_shapes(rows, cols, layout):
    lines, length = (rows, cols) if layout == ROWWISE else (cols, rows)
    assert length % 16 == 0, "blocked axis must be a multiple of 16"
    return (lines, length // 2), (lines, length // 16)


# ---------------------------------------------------------------- scalars

def bf16_to_f32(h: int) -> float:
    return lib().ref_bf16_to_f32(h)


def f32_to_bf16(f: float) -> int:
    return lib().ref_f32_to_bf16(f)


def e2m1_decode(code: int) -> float:
    return lib().ref_e2m1_decode(code)


def e2m1_rtn(y: float) -> int:
    return lib().ref_e2m1_rtn(y)


def e2m1_sr(y: float, u: float) -> int:
    return lib().ref_e2m1_sr(y, u)


def e4m3_decode(b: int) -> float:
    return lib().ref_e4m3_decode(b)


def e4m3_encode(x: float) -> int:
    return lib().ref_e4m3_encode(x)


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*ctr)
    k = (C.c_uint32 * 2)(*key)
    o = (C.c_uint32 * 4)()
    lib().ref_philox4x32_10(c, k, o)
    return tuple(int(v) for v in o)


def sr_uniform(seed: int, g: int) -> float:
    return lib().ref_sr_uniform(seed, g)


def rht_sign_word(seed: int, B: int) -> int:
    return lib().ref_rht_sign_word(seed, B)


def rht16(v, sign_word: int) -> np.ndarray:
    a = np.array(v, dtype=np.float32).copy()
    assert a.shape == (16,)
    lib().ref_rht16(_p(a, C.c_float), sign_word)
    return a


def block_scale(b: float, alpha: float, M: float) -> int:
    return lib().ref_block_scale(b, alpha, M)


def block_with_scale(v, alpha: float, S: int, rounding: int = RTN, u=None):
    """(E, codes[16], D[16]) of one block quantized with scale byte S."""
    a = np.array(v, dtype=np.float32).copy()
    assert a.shape == (16,)
    uu = np.zeros(16, np.float32) if u is None else np.array(u, dtype=np.float32).copy()
    q = np.zeros(16, np.uint8)
    D = np.zeros(16, np.float32)
    E = lib().ref_block_with_scale(_p(a, C.c_float), alpha, S, rounding, _p(uu, C.c_float),
                                   _p(q, C.c_uint8), _p(D, C.c_float))
    return float(E), q, D


def quantize_block(v, alpha: float, rounding: int = RTN, select: int = SEL_46_MSE, u=None):
    """4/6 on one block of up to 16 values (zero padded).  Returns a dict."""
    a = np.zeros(16, np.float32)
    a[:len(v)] = np.asarray(v, dtype=np.float32)
    uu = np.zeros(16, np.float32) if u is None else np.array(u, dtype=np.float32).copy()
    q = np.zeros(16, np.uint8)
    D = np.zeros(16, np.float32)
    S = C.c_uint8()
    four = C.c_uint8()
    E = np.zeros(2, np.float32)
    lib().ref_quantize_block(_p(a, C.c_float), alpha, rounding, select, _p(uu, C.c_float),
                             _p(q, C.c_uint8), _p(D, C.c_float), C.byref(S), C.byref(four),
                             _p(E, C.c_float))
    return {"codes": q, "D": D, "S": int(S.value), "four": int(four.value),
            "E6": float(E[0]), "E4": float(E[1])}


# ---------------------------------------------------------------- tensors

def tensor_scale(x_bits: np.ndarray, layout: int = ROWWISE, rht: int = 0, rht_seed: int = 0,
                 fp8_max: float = 256.0) -> float:
    rows, cols = _check_x(x_bits)
    _out_shapes(rows, cols, layout)
    a = C.c_float()
    fn, xp = _x(x_bits, "nvfp4_46_ref_tensor_scale")
    rc = fn(xp, rows, cols, layout, rht, rht_seed, fp8_max, C.byref(a))
    assert rc == 0
    return float(a.value)


def quantize(x_bits: np.ndarray, alpha: float, layout: int = ROWWISE, rounding: int = RTN,
             select: int = SEL_46_MSE, rht: int = 0, sr_seed: int = 0, rht_seed: int = 0,
             want_deq: bool = False):
    """Returns (codes, scales, choice[, deq_bits]) as uint8 / uint16 arrays."""
    rows, cols = _check_x(x_bits)
    cs, ss = _out_shapes(rows, cols, layout)
    codes = np.zeros(cs, np.uint8)
    scales = np.zeros(ss, np.uint8)
    choice = np.zeros(ss, np.uint8)
    deq = np.zeros((rows, cols), np.uint16) if want_deq else None
    fn, xp = _x(x_bits, "nvfp4_46_ref_quantize")
    rc = fn(xp, rows, cols, layout, rounding, select, rht, sr_seed, rht_seed, alpha,
            _p(codes, C.c_uint8), _p(scales, C.c_uint8), _p(choice, C.c_uint8),
            _p(deq, C.c_uint16))
    assert rc == 0
    return (codes, scales, choice, deq) if want_deq else (codes, scales, choice)


def quantize_rows(x_bits: np.ndarray, row0: int, alpha: float, layout: int = ROWWISE,
                  rounding: int = RTN, select: int = SEL_46_MSE, rht: int = 0, sr_seed: int = 0,
                  rht_seed: int = 0):
    """Quantize rows row0.. of a taller BF16 tensor (x_bits holds just those rows): the slice
    of the whole tensor's (codes, scales, choice, deq)."""
    assert x_bits.dtype == np.uint16 and row0 % 16 == 0
    rows, cols = _check_x(x_bits)
    cs, ss = _out_shapes(rows, cols, layout)
    codes, scales, choice = np.zeros(cs, np.uint8), np.zeros(ss, np.uint8), np.zeros(ss, np.uint8)
    deq = np.zeros((rows, cols), np.uint16)
    rc = lib().nvfp4_46_ref_quantize_rows(_p(x_bits, C.c_uint16), rows, cols, row0, layout,
                                          rounding, select, rht, sr_seed, rht_seed, alpha,
                                          _p(codes, C.c_uint8), _p(scales, C.c_uint8),
                                          _p(choice, C.c_uint8), _p(deq, C.c_uint16))
    assert rc == 0
    return codes, scales, choice, deq


def dequantize(codes: np.ndarray, scales: np.ndarray, alpha: float, rows: int, cols: int,
               layout: int = ROWWISE) -> np.ndarray:
    cs, ss = _out_shapes(rows, cols, layout)
    assert codes.shape == cs and scales.shape == ss
    assert codes.dtype == np.uint8 and scales.dtype == np.uint8
    out = np.zeros((rows, cols), np.uint16)
    rc = lib().nvfp4_46_ref_dequantize(_p(codes, C.c_uint8), _p(scales, C.c_uint8), alpha, rows,
                                       cols, layout, _p(out, C.c_uint16))
    assert rc == 0
    return out


def fake_quant(x_bits: np.ndarray, alpha: float, layout: int = ROWWISE, rounding: int = RTN,
               select: int = SEL_46_MSE, rht: int = 0, sr_seed: int = 0,
               rht_seed: int = 0) -> np.ndarray:
    rows, cols = _check_x(x_bits)
    _out_shapes(rows, cols, layout)
    out = np.zeros((rows, cols), np.uint16)
    if x_bits.dtype == np.float32:
        rc = lib().nvfp4_46_ref_quantize_f32(_p(x_bits, C.c_float), rows, cols, layout, rounding,
                                             select, rht, sr_seed, rht_seed, alpha, None, None,
                                             None, _p(out, C.c_uint16))
    else:
        rc = lib().nvfp4_46_ref_fake_quant(_p(x_bits, C.c_uint16), rows, cols, layout, rounding,
                                           select, rht, sr_seed, rht_seed, alpha,
                                           _p(out, C.c_uint16))
    assert rc == 0
    return out


def block_abs_metric(v, D, select: int) -> float:
    a = np.array(v, dtype=np.float32).copy()
    d = np.array(D, dtype=np.float32).copy()
    assert a.shape == (16,) and d.shape == (16,)
    return float(lib().ref_block_abs_metric(_p(a, C.c_float), _p(d, C.c_float), select))


def block_errors(x_bits: np.ndarray, alpha: float, layout: int = ROWWISE, rounding: int = RTN,
                 rht: int = 0, sr_seed: int = 0, rht_seed: int = 0, select: int = SEL_46_MSE):
    assert x_bits.dtype == np.uint16
    rows, cols = _check_x(x_bits)
    _, ss = _out_shapes(rows, cols, layout)
    E6 = np.zeros(ss, np.float32)
    E4 = np.zeros(ss, np.float32)
    rc = lib().nvfp4_46_ref_block_errors_sel(_p(x_bits, C.c_uint16), rows, cols, layout, rounding,
                                             select, rht, sr_seed, rht_seed, alpha,
                                             _p(E6, C.c_float), _p(E4, C.c_float))
    assert rc == 0
    return E6, E4


def quantize_2d(x_bits: np.ndarray, alpha: float, rounding: int = RTN, select: int = SEL_46_MSE,
                sr_seed: int = 0):
    """16x16-tile quantization: (codes [rows][cols/2], scales, choice [rows/16][cols/16], deq)."""
    rows, cols = _check_x(x_bits)
    assert rows % 16 == 0 and cols % 16 == 0
    codes = np.zeros((rows, cols // 2), np.uint8)
    scales = np.zeros((rows // 16, cols // 16), np.uint8)
    choice = np.zeros((rows // 16, cols // 16), np.uint8)
    deq = np.zeros((rows, cols), np.uint16)
    fn, xp = _x(x_bits, "nvfp4_46_ref_quantize_2d")
    rc = fn(xp, rows, cols, rounding, select, sr_seed, alpha, _p(codes, C.c_uint8),
            _p(scales, C.c_uint8), _p(choice, C.c_uint8), _p(deq, C.c_uint16))
    assert rc == 0
    return codes, scales, choice, deq


def repack_2d_columnwise(codes: np.ndarray, scales: np.ndarray, choice: np.ndarray):
    """Row-packed 2D-block outputs -> the transposed matrix's packing:
    (codes_col [cols][rows/2], scales_col, choice_col [cols/16][rows/16])."""
    rows, cols = codes.shape[0], codes.shape[1] * 2
    assert scales.shape == (rows // 16, cols // 16) and choice.shape == scales.shape
    cc = np.zeros((cols, rows // 2), np.uint8)
    sc = np.zeros((cols // 16, rows // 16), np.uint8)
    fc = np.zeros((cols // 16, rows // 16), np.uint8)
    rc = lib().nvfp4_46_ref_repack_2d_columnwise(_p(codes, C.c_uint8), _p(scales, C.c_uint8),
                                                 _p(choice, C.c_uint8), rows, cols,
                                                 _p(cc, C.c_uint8), _p(sc, C.c_uint8),
                                                 _p(fc, C.c_uint8))
    assert rc == 0
    return cc, sc, fc


def dequantize_2d_columnwise(codes_col: np.ndarray, scales_col: np.ndarray, alpha: float,
                             rows: int, cols: int) -> np.ndarray:
    assert codes_col.shape == (cols, rows // 2) and scales_col.shape == (cols // 16, rows // 16)
    out = np.zeros((rows, cols), np.uint16)
    rc = lib().nvfp4_46_ref_dequantize_2d_columnwise(_p(codes_col, C.c_uint8),
                                                     _p(scales_col, C.c_uint8), alpha, rows, cols,
                                                     _p(out, C.c_uint16))
    assert rc == 0
    return out


def dequantize_2d(codes: np.ndarray, scales: np.ndarray, alpha: float, rows: int,
                  cols: int) -> np.ndarray:
    assert codes.shape == (rows, cols // 2) and scales.shape == (rows // 16, cols // 16)
    out = np.zeros((rows, cols), np.uint16)
    rc = lib().nvfp4_46_ref_dequantize_2d(_p(codes, C.c_uint8), _p(scales, C.c_uint8), alpha, rows,
                                          cols, _p(out, C.c_uint16))
    assert rc == 0
    return out


def gemm(codes_a: np.ndarray, scales_a: np.ndarray, alpha_a: float, codes_b: np.ndarray,
         scales_b: np.ndarray, alpha_b: float, want_abs: bool = False, tiles_a: bool = False,
         tiles_b: bool = False):
    """C [M][N] (float64) = alpha_a * alpha_b * A . B^T of two rowwise NVFP4 operands
    (codes [M][K/2] / [N][K/2], scales [M][K/16] / [N][K/16], or [rows/16][K/16] for an
    operand quantized with 16x16 tiles); with `want_abs` also the same sum over the products'
    magnitudes."""
    M, N = codes_a.shape[0], codes_b.shape[0]
    K = codes_a.shape[1] * 2
    assert codes_b.shape == (N, K // 2) and K % 16 == 0
    assert scales_a.shape == ((M // 16 if tiles_a else M), K // 16)
    assert scales_b.shape == ((N // 16 if tiles_b else N), K // 16)
    for a in (codes_a, scales_a, codes_b, scales_b):
        assert a.dtype == np.uint8
    out = np.zeros((M, N), np.float64)
    out_abs = np.zeros((M, N), np.float64) if want_abs else None
    rc = lib().nvfp4_46_ref_gemm(_p(codes_a, C.c_uint8), _p(scales_a, C.c_uint8), alpha_a,
                                 _p(codes_b, C.c_uint8), _p(scales_b, C.c_uint8), alpha_b, M, N, K,
                                 int(tiles_a), int(tiles_b), _p(out, C.c_double),
                                 _p(out_abs, C.c_double))
    assert rc == 0
    return (out, out_abs) if want_abs else out


def e2m1_rtn_bits_range(first_bits: int, n: int) -> np.ndarray:
    out = np.zeros(n, np.uint8)
    lib().ref_e2m1_rtn_bits_range(first_bits, n, _p(out, C.c_uint8))
    return out


def e2m1_sr_bits_range(first_bits: int, n: int, u: float) -> np.ndarray:
    """e2m1_sr of the n fp32 values with bit patterns first_bits .. first_bits + n - 1, all
    with the uniform u."""
    out = np.empty(n, dtype=np.uint8)
    lib().ref_e2m1_sr_bits_range(first_bits, n, u, _p(out, C.c_uint8))
    return out


def e2m1_sr_n(y: np.ndarray, u: np.ndarray) -> np.ndarray:
    """e2m1_sr of n (y, u) pairs (float32 arrays)."""
    y = np.ascontiguousarray(y, dtype=np.float32)
    u = np.ascontiguousarray(u, dtype=np.float32)
    assert y.shape == u.shape
    out = np.empty(y.size, dtype=np.uint8)
    lib().ref_e2m1_sr_n(_p(y, C.c_float), _p(u, C.c_float), y.size, _p(out, C.c_uint8))
    return out


def e4m3_encode_bits_range(first_bits: int, n: int) -> np.ndarray:
    out = np.zeros(n, np.uint8)
    lib().ref_e4m3_encode_bits_range(first_bits, n, _p(out, C.c_uint8))
    return out
