"""The kernels' per-block code compiled for the host (tests/host_model/), behind ctypes.

Test infrastructure.  ``csrc/block.hpp`` and ``csrc/codec.hpp`` -- the code every quantizing
kernel runs per block -- are compiled with the host compiler, the gfx950 conversion
instructions replaced by plain definitions of what they compute, so that CPU tests can put
the GPU path's block logic next to the oracle on inputs of any range without a GPU.
"""
from __future__ import annotations

import ctypes as C
import os
import shutil
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent / "host_model"
_ROOT = _HERE.parent.parent
_CSRC = _ROOT / "paper_2512_02010_amd" / "csrc"
_SO = _HERE / "_build" / "libhost_model.so"
_SOURCES = [_HERE / "model.cpp", _HERE / "gfx950_on_host.hpp", _CSRC / "block.hpp", _CSRC / "codec.hpp"]

RTN, SR, SR_AFTER_RTN_SELECT = 0, 1, 2


def _compiler() -> str:
    for cand in ("/opt/rocm/llvm/bin/clang++", shutil.which("amdclang++"), shutil.which("clang++")):
        if cand and Path(cand).exists():
            return cand
    raise RuntimeError("no clang++ found (the headers use clang vector extensions)")


def build(force: bool = False) -> Path:
    newest = max(p.stat().st_mtime for p in _SOURCES)
    if _SO.exists() and not force and _SO.stat().st_mtime >= newest:
        return _SO
    _SO.parent.mkdir(parents=True, exist_ok=True)
    tmp = _SO.with_suffix(f".tmp{os.getpid()}.so")
    # one rounding per operation, as in the device build; no fast-math, denormals kept
    subprocess.run([_compiler(), "-x", "c++", "-std=c++17", "-O1", "-fPIC", "-shared",
                    "-ffp-contract=off", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
                    f"-I{_CSRC}", f"-I{_ROOT / 'include'}", str(_HERE / "model.cpp"), "-o", str(tmp)],
                   check=True)
    os.replace(tmp, _SO)
    return _SO


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        L = C.CDLL(str(build()))
        f32p, u32p, u8p = C.POINTER(C.c_float), C.POINTER(C.c_uint32), C.POINTER(C.c_uint8)
        L.hm_quantize_blocks.restype = None
        L.hm_quantize_blocks.argtypes = [f32p, f32p, C.c_int64, C.c_float, C.c_int, C.c_int, u32p,
                                         u8p, u8p]
        L.hm_second_passes.restype = C.c_int
        L.hm_second_passes.argtypes = []
        L.hm_tile_decision.restype = C.c_int
        L.hm_tile_decision.argtypes = [f32p, f32p, C.c_float, C.c_int, u8p, u8p, C.POINTER(C.c_int)]
        L.hm_e2m1_sr.restype = None
        L.hm_e2m1_sr.argtypes = [f32p, f32p, C.c_int64, u8p, u8p]
        L.hm_block_scale.restype = C.c_int
        L.hm_block_scale.argtypes = [C.c_float, C.c_float, C.c_int, C.c_int]
        L.hm_philox.restype = None
        L.hm_philox.argtypes = [u32p, C.c_uint32, C.c_uint32, u32p]
        L.hm_rht16.restype = None
        L.hm_rht16.argtypes = [f32p, C.c_uint32]
        _lib = L
    return _lib


def _p(a, ctype):
    return None if a is None else a.ctypes.data_as(C.POINTER(ctype))


def quantize_blocks(v: np.ndarray, alpha: float, rounding: int = RTN, select: int = 0,
                    u: np.ndarray | None = None):
    """v: [n][16] float32 (u likewise, for stochastic rounding).  Returns (codes [n][8] uint8
    in the library's nibble order, scale bytes [n], choices [n])."""
    v = np.ascontiguousarray(v, dtype=np.float32)
    n = v.shape[0]
    assert v.shape == (n, 16)
    if u is not None:
        u = np.ascontiguousarray(u, dtype=np.float32)
        assert u.shape == v.shape
    codes = np.zeros((n, 2), np.uint32)
    scale = np.zeros(n, np.uint8)
    four = np.zeros(n, np.uint8)
    lib().hm_quantize_blocks(_p(v, C.c_float), _p(u, C.c_float), n, alpha, rounding, select,
                             _p(codes, C.c_uint32), _p(scale, C.c_uint8), _p(four, C.c_uint8))
    return codes.view(np.uint8).reshape(n, 8), scale, four


def second_passes() -> int:
    """Blocks so far that the estimate pass could not decide (redone with the defined errors)."""
    return lib().hm_second_passes()


def tile_decision(v: np.ndarray, alpha: float, rounding: int = RTN, u: np.ndarray | None = None):
    """v: [16][16] float32, one tile.  Returns (four, scale6, scale4, took_defined_path)."""
    v = np.ascontiguousarray(v, dtype=np.float32)
    assert v.shape == (16, 16)
    if u is not None:
        u = np.ascontiguousarray(u, dtype=np.float32)
    s6, s4, path = C.c_uint8(), C.c_uint8(), C.c_int()
    four = lib().hm_tile_decision(_p(v, C.c_float), _p(u, C.c_float), alpha, rounding, C.byref(s6),
                                  C.byref(s4), C.byref(path))
    return four, s6.value, s4.value, path.value


def e2m1_sr(y: np.ndarray, u: np.ndarray):
    """(codes by the software rule, codes by the conversion instruction | 0x80 where the
    kernels would redo the block in software)."""
    y = np.ascontiguousarray(y, dtype=np.float32)
    u = np.ascontiguousarray(u, dtype=np.float32)
    out = np.zeros(y.shape, np.uint8)
    fast = np.zeros(y.shape, np.uint8)
    lib().hm_e2m1_sr(_p(y, C.c_float), _p(u, C.c_float), y.size, _p(out, C.c_uint8), _p(fast, C.c_uint8))
    return out, fast


def block_scale(b: float, alpha: float, M: int) -> int:
    """The byte for one M as the always-6 / always-4 kernels compute it."""
    return lib().hm_block_scale(b, alpha, M, 0)


def block_scale_pair(b: float, alpha: float):
    """(S6, S4) as the 4/6 kernels compute them, in one go."""
    r = lib().hm_block_scale(b, alpha, 6, 1)
    return r & 0xFF, r >> 8


def philox(ctr, key):
    c = (C.c_uint32 * 4)(*ctr)
    o = (C.c_uint32 * 4)()
    lib().hm_philox(c, key[0], key[1], o)
    return tuple(int(x) for x in o)


def rht16(v, sign_word: int) -> np.ndarray:
    a = np.array(v, dtype=np.float32).copy()
    lib().hm_rht16(_p(a, C.c_float), sign_word)
    return a
