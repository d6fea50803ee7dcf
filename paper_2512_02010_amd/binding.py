"""Thin Python binding of ``libnvfp4_46.so`` (ctypes; argument marshalling only).

Every function has the name of the C entry point it calls (``include/nvfp4_46.h``)
and does no arithmetic of its own.  PyTorch supplies device memory and the
stream; tensors passed in must live on the current CUDA (ROCm) device.  There
is no CPU fallback: if the shared library has not been built, loading fails.
"""
from __future__ import annotations

import ctypes as C
import os
from pathlib import Path

import torch

_PKG = Path(__file__).resolve().parent

ROWWISE, COLWISE, BOTH = 1, 2, 3
BLOCK2D = 4          # nvfp4_46_dequantize's layout value for 16x16-tile data
RTN, SR, SR_AFTER_RTN_SELECT = 0, 1, 2
SEL_46_MSE, SEL_FORCE6, SEL_FORCE4, SEL_46_MAE, SEL_46_ABSMAX = 0, 1, 2, 3, 4
X_BF16, X_F32 = 0, 1
OUT_BF16, OUT_F32 = 0, 1
GEMM_A_TILE_SCALES, GEMM_B_TILE_SCALES = 1, 2

STATUS_NAMES = {0: "NVFP4_OK", 1: "NVFP4_ERR_NULL", 2: "NVFP4_ERR_SHAPE", 3: "NVFP4_ERR_ALIGN",
                4: "NVFP4_ERR_PARAM", 5: "NVFP4_ERR_UNSUPPORTED", 6: "NVFP4_ERR_HIP"}

EXPORTS = (
    "nvfp4_46_tensor_scale", "nvfp4_46_tensor_scale_ws", "nvfp4_46_tensor_scale_static",
    "nvfp4_46_quantize", "nvfp4_46_dequantize", "nvfp4_46_fake_quant",
    "nvfp4_46_gemm", "nvfp4_46_status_string", "nvfp4_46_debug_e2m1_rtn_range", "nvfp4_46_debug_e4m3_range",
    "nvfp4_46_debug_decode_tables", "nvfp4_46_debug_bf16_range", "nvfp4_46_debug_e2m1_sr",
    "nvfp4_46_debug_philox",
)


class Params(C.Structure):
    """Mirror of ``nvfp4_46_params``."""
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64), ("layout", C.c_uint32),
                ("rounding", C.c_uint32), ("select", C.c_uint32), ("rht", C.c_uint32),
                ("sr_seed", C.c_uint64), ("rht_seed", C.c_uint64), ("fp8_max", C.c_float),
                ("block2d", C.c_uint32), ("x_dtype", C.c_uint32)]


class Nvfp4Error(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)} ({status_string(status)})")


def library_path() -> Path:
    return Path(os.environ.get("NVFP4_46_LIB", _PKG / "libnvfp4_46.so"))


_lib = None


def lib() -> C.CDLL:
    """Load the HIP library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        path = library_path()
        if not path.exists():
            raise FileNotFoundError(
                f"{path} is missing: build it with `python -m paper_2512_02010_amd.build` "
                "(there is no CPU fallback)")
        L = C.CDLL(str(path))
        vp, i64, u32, u64 = C.c_void_p, C.c_int64, C.c_uint32, C.c_uint64
        pp = C.POINTER(Params)
        L.nvfp4_46_tensor_scale.restype = C.c_int
        L.nvfp4_46_tensor_scale.argtypes = [vp, pp, vp, vp]
        L.nvfp4_46_tensor_scale_ws.restype = C.c_int
        L.nvfp4_46_tensor_scale_ws.argtypes = [vp, pp, vp, vp, C.c_size_t, vp]
        L.nvfp4_46_tensor_scale_static.restype = C.c_int
        L.nvfp4_46_tensor_scale_static.argtypes = [vp, pp, vp, vp]
        L.nvfp4_46_quantize.restype = C.c_int
        L.nvfp4_46_quantize.argtypes = [vp, pp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.nvfp4_46_dequantize.restype = C.c_int
        L.nvfp4_46_dequantize.argtypes = [vp, vp, vp, i64, i64, u32, vp, vp]
        L.nvfp4_46_fake_quant.restype = C.c_int
        L.nvfp4_46_fake_quant.argtypes = [vp, pp, vp, vp, vp]
        L.nvfp4_46_gemm.restype = C.c_int
        L.nvfp4_46_gemm.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, u32, u32, vp, vp]
        L.nvfp4_46_status_string.restype = C.c_char_p
        L.nvfp4_46_status_string.argtypes = [C.c_int]
        L.nvfp4_46_debug_e2m1_rtn_range.restype = C.c_int
        L.nvfp4_46_debug_e2m1_rtn_range.argtypes = [u32, i64, vp, vp]
        L.nvfp4_46_debug_e4m3_range.restype = C.c_int
        L.nvfp4_46_debug_e4m3_range.argtypes = [u32, i64, vp, vp]
        L.nvfp4_46_debug_decode_tables.restype = C.c_int
        L.nvfp4_46_debug_decode_tables.argtypes = [vp, vp]
        L.nvfp4_46_debug_bf16_range.restype = C.c_int
        L.nvfp4_46_debug_bf16_range.argtypes = [u32, u32, i64, vp, vp]
        L.nvfp4_46_debug_e2m1_sr.restype = C.c_int
        L.nvfp4_46_debug_e2m1_sr.argtypes = [vp, vp, i64, vp, vp, vp]
        L.nvfp4_46_debug_philox.restype = C.c_int
        L.nvfp4_46_debug_philox.argtypes = [vp, u32, u32, i64, vp, vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().nvfp4_46_status_string(int(status)).decode()


def make_params(rows: int, cols: int, layout: int = ROWWISE, rounding: int = RTN,
                select: int = SEL_46_MSE, rht: int = 0, sr_seed: int = 0, rht_seed: int = 0,
                fp8_max: float = 256.0, block2d: int = 0, x_dtype: int = X_BF16) -> Params:
    return Params(rows, cols, layout, rounding, select, rht, sr_seed, rht_seed, fp8_max, block2d,
                  x_dtype)


def _device_empty(shape, dtype, device) -> torch.Tensor:
    return torch.empty(shape, dtype=dtype, device=device)


# Every output tensor the helpers below create comes from this callable (shape, dtype,
# device) -> tensor.  The GPU tests swap in an allocator that places each output inside a
# larger sentinel-filled buffer and checks afterwards that nothing wrote past its ends.
OUTPUT_ALLOCATOR = _device_empty


def _new(shape, dtype, device) -> torch.Tensor:
    return OUTPUT_ALLOCATOR(shape, dtype, device)


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    assert t.is_cuda and t.is_contiguous(), "tensors must be contiguous device tensors"
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _check(rc: int, where: str):
    if rc != 0:
        raise Nvfp4Error(rc, where)


# ---- raw entry points (return the status code; used by the error-path tests) -------------

def tensor_scale_raw(x, params: Params, alpha, stream=None) -> int:
    return lib().nvfp4_46_tensor_scale(_ptr(x), C.byref(params) if params is not None else None,
                                       _ptr(alpha), _stream(stream))


TENSOR_SCALE_WS_BYTES = 4352


def tensor_scale_ws_raw(x, params: Params, alpha, workspace, workspace_bytes: int, stream=None) -> int:
    return lib().nvfp4_46_tensor_scale_ws(_ptr(x), C.byref(params) if params is not None else None,
                                          _ptr(alpha), _ptr(workspace), workspace_bytes,
                                          _stream(stream))


def tensor_scale_static_raw(x, params: Params, alpha, stream=None) -> int:
    return lib().nvfp4_46_tensor_scale_static(_ptr(x), C.byref(params) if params is not None else None,
                                              _ptr(alpha), _stream(stream))


def quantize_raw(x, params, alpha, codes_row, scales_row, codes_col, scales_col, choice_row,
                 choice_col, stream=None) -> int:
    return lib().nvfp4_46_quantize(_ptr(x), C.byref(params) if params is not None else None,
                                   _ptr(alpha), _ptr(codes_row), _ptr(scales_row), _ptr(codes_col),
                                   _ptr(scales_col), _ptr(choice_row), _ptr(choice_col),
                                   _stream(stream))


def dequantize_raw(codes, scales, alpha, rows, cols, layout, out, stream=None) -> int:
    return lib().nvfp4_46_dequantize(_ptr(codes), _ptr(scales), _ptr(alpha), rows, cols, layout,
                                     _ptr(out), _stream(stream))


def fake_quant_raw(x, params, alpha, out, stream=None) -> int:
    return lib().nvfp4_46_fake_quant(_ptr(x), C.byref(params) if params is not None else None,
                                     _ptr(alpha), _ptr(out), _stream(stream))


def gemm_raw(codes_a, scales_a, alpha_a, codes_b, scales_b, alpha_b, M, N, K, out_dtype, out,
             stream=None, flags: int = 0) -> int:
    return lib().nvfp4_46_gemm(_ptr(codes_a), _ptr(scales_a), _ptr(alpha_a), _ptr(codes_b),
                               _ptr(scales_b), _ptr(alpha_b), M, N, K, out_dtype, flags,
                               _ptr(out), _stream(stream))


# ---- the same calls with output allocation and error checking ---------------------------

def _shape_of(x):
    assert x.dim() == 2 and x.dtype in (torch.bfloat16, torch.float32)
    return int(x.shape[0]), int(x.shape[1])


def x_dtype_of(x: torch.Tensor) -> int:
    return X_F32 if x.dtype == torch.float32 else X_BF16


def nvfp4_46_tensor_scale(x: torch.Tensor, layout: int = ROWWISE, rht: int = 0, rht_seed: int = 0,
                          fp8_max: float = 256.0, out: torch.Tensor | None = None,
                          stream=None) -> torch.Tensor:
    """alpha (1-element fp32 device tensor) of a BF16 or fp32 device tensor."""
    rows, cols = _shape_of(x)
    alpha = out if out is not None else _new((1,), torch.float32, x.device)
    p = make_params(rows, cols, layout=layout, rht=rht, rht_seed=rht_seed, fp8_max=fp8_max,
                    x_dtype=x_dtype_of(x))
    _check(tensor_scale_raw(x, p, alpha, stream), "nvfp4_46_tensor_scale")
    return alpha


def new_workspace(device="cuda") -> torch.Tensor:
    """A zeroed workspace for nvfp4_46_tensor_scale_ws (the calls leave it zeroed)."""
    return torch.zeros(TENSOR_SCALE_WS_BYTES, dtype=torch.uint8, device=device)


def nvfp4_46_tensor_scale_ws(x: torch.Tensor, workspace: torch.Tensor, layout: int = ROWWISE,
                             rht: int = 0, rht_seed: int = 0, fp8_max: float = 256.0,
                             out: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """nvfp4_46_tensor_scale in one launch, with a caller-owned zeroed workspace."""
    rows, cols = _shape_of(x)
    alpha = out if out is not None else _new((1,), torch.float32, x.device)
    p = make_params(rows, cols, layout=layout, rht=rht, rht_seed=rht_seed, fp8_max=fp8_max,
                    x_dtype=x_dtype_of(x))
    _check(tensor_scale_ws_raw(x, p, alpha, workspace, workspace.numel(), stream),
           "nvfp4_46_tensor_scale_ws")
    return alpha


def alloc_outputs(rows: int, cols: int, layout: int, device, want_choice: bool = True,
                  block2d: int = 0) -> dict:
    """uint8 device tensors for nvfp4_46_quantize's outputs in the requested layout(s)."""
    o = dict.fromkeys(("codes_row", "scales_row", "choice_row", "codes_col", "scales_col",
                       "choice_col"))
    def u8(shape):
        return _new(shape, torch.uint8, device)

    if layout & ROWWISE:
        srows = rows // 16 if block2d else rows
        o["codes_row"] = u8((rows, cols // 2))
        o["scales_row"] = u8((srows, cols // 16))
        if want_choice:
            o["choice_row"] = u8((srows, cols // 16))
    if layout & COLWISE:
        scols = cols // 16 if block2d else cols
        o["codes_col"] = u8((cols, rows // 2))
        o["scales_col"] = u8((scols, rows // 16))
        if want_choice:
            o["choice_col"] = u8((scols, rows // 16))
    return o


def nvfp4_46_quantize(x: torch.Tensor, alpha: torch.Tensor, layout: int = ROWWISE,
                      rounding: int = RTN, select: int = SEL_46_MSE, rht: int = 0,
                      sr_seed: int = 0, rht_seed: int = 0, fp8_max: float = 256.0,
                      want_choice: bool = True, out: dict | None = None, stream=None,
                      block2d: int = 0) -> dict:
    rows, cols = _shape_of(x)
    o = out if out is not None else alloc_outputs(rows, cols, layout, x.device, want_choice,
                                                  block2d)
    p = make_params(rows, cols, layout, rounding, select, rht, sr_seed, rht_seed, fp8_max,
                    block2d, x_dtype_of(x))
    _check(quantize_raw(x, p, alpha, o["codes_row"], o["scales_row"], o["codes_col"],
                        o["scales_col"], o["choice_row"], o["choice_col"], stream),
           "nvfp4_46_quantize")
    return o


def nvfp4_46_dequantize(codes: torch.Tensor, scales: torch.Tensor, alpha: torch.Tensor, rows: int,
                        cols: int, layout: int = ROWWISE, out: torch.Tensor | None = None,
                        stream=None) -> torch.Tensor:
    if out is None:
        out = _new((rows, cols), torch.bfloat16, codes.device)
    _check(dequantize_raw(codes, scales, alpha, rows, cols, layout, out, stream),
           "nvfp4_46_dequantize")
    return out


def nvfp4_46_fake_quant(x: torch.Tensor, alpha: torch.Tensor, layout: int = ROWWISE,
                        rounding: int = RTN, select: int = SEL_46_MSE, rht: int = 0,
                        sr_seed: int = 0, rht_seed: int = 0, fp8_max: float = 256.0,
                        out: torch.Tensor | None = None, stream=None,
                        block2d: int = 0) -> torch.Tensor:
    rows, cols = _shape_of(x)
    if out is None:
        out = _new(tuple(x.shape), torch.bfloat16, x.device)
    p = make_params(rows, cols, layout, rounding, select, rht, sr_seed, rht_seed, fp8_max,
                    block2d, x_dtype_of(x))
    _check(fake_quant_raw(x, p, alpha, out, stream), "nvfp4_46_fake_quant")
    return out


def nvfp4_46_gemm(codes_a: torch.Tensor, scales_a: torch.Tensor, alpha_a: torch.Tensor,
                  codes_b: torch.Tensor, scales_b: torch.Tensor, alpha_b: torch.Tensor,
                  out_dtype: int = OUT_BF16, out: torch.Tensor | None = None,
                  stream=None, flags: int = 0) -> torch.Tensor:
    """C [M][N] = alpha_a alpha_b A B^T of two rowwise-quantized operands A [M][K], B [N][K];
    `flags` marks operands whose scales come per 16x16 tile ([rows/16][K/16])."""
    M, N, K = int(codes_a.shape[0]), int(codes_b.shape[0]), int(codes_a.shape[1]) * 2
    assert codes_b.shape[1] * 2 == K
    assert tuple(scales_a.shape) == (M // 16 if flags & GEMM_A_TILE_SCALES else M, K // 16)
    assert tuple(scales_b.shape) == (N // 16 if flags & GEMM_B_TILE_SCALES else N, K // 16)
    if out is None:
        out = _new((M, N), torch.float32 if out_dtype == OUT_F32 else torch.bfloat16, codes_a.device)
    _check(gemm_raw(codes_a, scales_a, alpha_a, codes_b, scales_b, alpha_b, M, N, K, out_dtype,
                    out, stream, flags), "nvfp4_46_gemm")
    return out


# ---- scalar codecs ------------------------------------------------------------------------

def nvfp4_46_debug_e2m1_rtn_range(first_bits: int, n: int, device="cuda") -> torch.Tensor:
    out = torch.empty(n, dtype=torch.uint8, device=device)
    _check(lib().nvfp4_46_debug_e2m1_rtn_range(first_bits, n, _ptr(out), _stream(None)),
           "nvfp4_46_debug_e2m1_rtn_range")
    return out


def nvfp4_46_debug_e4m3_range(first_bits: int, n: int, device="cuda") -> torch.Tensor:
    out = torch.empty(n, dtype=torch.uint8, device=device)
    _check(lib().nvfp4_46_debug_e4m3_range(first_bits, n, _ptr(out), _stream(None)),
           "nvfp4_46_debug_e4m3_range")
    return out


def nvfp4_46_debug_decode_tables(device="cuda") -> torch.Tensor:
    out = torch.empty(272, dtype=torch.float32, device=device)
    _check(lib().nvfp4_46_debug_decode_tables(_ptr(out), _stream(None)),
           "nvfp4_46_debug_decode_tables")
    return out


def nvfp4_46_debug_bf16_range(first_bits: int, stride: int, n: int, device="cuda") -> torch.Tensor:
    out = torch.empty(n, dtype=torch.int16, device=device)
    _check(lib().nvfp4_46_debug_bf16_range(first_bits, stride, n, _ptr(out), _stream(None)),
           "nvfp4_46_debug_bf16_range")
    return out


def nvfp4_46_debug_e2m1_sr(y: torch.Tensor, words: torch.Tensor):
    """(codes by the software rule, codes by the conversion instruction with bit 7 = not trusted)
    for fp32 values `y` and int32 random words `words` (uniform = top 24 bits)."""
    assert y.dtype == torch.float32 and words.dtype == torch.int32 and y.numel() == words.numel()
    out = _new(y.numel(), dtype=torch.uint8, device=y.device)
    fast = _new(y.numel(), dtype=torch.uint8, device=y.device)
    _check(lib().nvfp4_46_debug_e2m1_sr(_ptr(y), _ptr(words), y.numel(), _ptr(out), _ptr(fast),
                                        _stream(None)), "nvfp4_46_debug_e2m1_sr")
    return out, fast


def nvfp4_46_debug_philox(ctr: torch.Tensor, key0: int, key1: int) -> torch.Tensor:
    assert ctr.dtype == torch.int32 and ctr.dim() == 2 and ctr.shape[1] == 4
    out = torch.empty_like(ctr)
    _check(lib().nvfp4_46_debug_philox(_ptr(ctr), key0, key1, ctr.shape[0], _ptr(out),
                                       _stream(None)), "nvfp4_46_debug_philox")
    return out
