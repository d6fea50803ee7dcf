"""CPU-side checks of the C-ABI library: it loads, exports what the header declares,
and its host-side argument validation returns the documented codes without touching
the GPU (every call below fails validation before any HIP call)."""
import ctypes as C
import re
from pathlib import Path

import pytest

from paper_2512_02010_amd import binding as B

ROOT = Path(__file__).resolve().parent.parent
HEADER = (ROOT / "include" / "nvfp4_46.h").read_text()


def _declared():
    names = re.findall(r"^(?:int|const char \*)\s*(nvfp4_46_\w+)\s*\(", HEADER, flags=re.M)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = _declared()
    assert len(names) == 14
    assert sorted(B.EXPORTS) == names
    for n in names:
        assert hasattr(L, n), n


def test_params_struct_layout_matches_header():
    assert C.sizeof(B.Params) == 64
    offs = {f[0]: getattr(B.Params, f[0]).offset for f in B.Params._fields_}
    assert offs == {"rows": 0, "cols": 8, "layout": 16, "rounding": 20, "select": 24, "rht": 28,
                    "sr_seed": 32, "rht_seed": 40, "fp8_max": 48, "block2d": 52,
                    "x_dtype": 56}
    # enum values quoted in the header
    for name, val in (("NVFP4_ROWWISE", 1), ("NVFP4_COLWISE", 2), ("NVFP4_RTN", 0), ("NVFP4_SR", 1), ("NVFP4_SR_AFTER_RTN_SELECT", 2),
                      ("NVFP4_SEL_46_MSE", 0), ("NVFP4_SEL_FORCE6", 1), ("NVFP4_SEL_FORCE4", 2),
                      ("NVFP4_SEL_46_MAE", 3), ("NVFP4_SEL_46_ABSMAX", 4), ("NVFP4_X_BF16", 0),
                      ("NVFP4_X_F32", 1)):
        assert re.search(rf"{name} = {val}\b", HEADER), name


def test_status_strings():
    for code in range(7):
        s = B.status_string(code)
        assert isinstance(s, str) and s
    assert B.status_string(0) == "ok" and "unknown" in B.status_string(99)


P = 0x10000      # a fake, 16-byte aligned, never dereferenced "device pointer"


def _q(params, x=P, alpha=P, cr=P, sr=P, cc=None, sc=None, hr=None, hc=None):
    return B.quantize_raw(x, params, alpha, cr, sr, cc, sc, hr, hc, stream=0)


def test_quantize_validation_codes():
    ok = B.make_params(32, 64)
    assert _q(None) == 1 and _q(ok, x=None) == 1 and _q(ok, alpha=None) == 1
    assert _q(ok, cr=None) == 1 and _q(ok, sr=None) == 1
    assert _q(B.make_params(0, 64)) == 2 and _q(B.make_params(32, -16)) == 2
    assert _q(B.make_params(32, 72)) == 2                       # cols % 16 != 0, rowwise
    assert _q(B.make_params(40, 64, layout=B.COLWISE), cr=None, sr=None, cc=P, sc=P) == 2
    assert _q(B.make_params(32, 36, layout=B.COLWISE), cr=None, sr=None, cc=P, sc=P) == 2
    assert _q(ok, x=P + 2) == 3 and _q(ok, cr=P + 8) == 3 and _q(ok, hr=P + 1) == 3
    assert _q(B.make_params(32, 64, layout=0)) == 4 and _q(B.make_params(32, 64, layout=4)) == 4
    assert _q(B.make_params(32, 64, rounding=3)) == 4 and _q(B.make_params(32, 64, select=5)) == 4
    assert _q(B.make_params(32, 64, rht=2)) == 4
    assert _q(B.make_params(32, 64, x_dtype=2)) == 4
    assert _q(B.make_params(32, 64, fp8_max=0.0)) == 4
    assert _q(B.make_params(32, 64, fp8_max=449.0)) == 4
    assert _q(B.make_params(32, 64, fp8_max=float("nan"))) == 4
    bad = B.make_params(32, 64)
    bad.block2d = 2
    assert _q(bad) == 4
    # 16x16 tiles: both dims multiples of 16, no transform
    assert _q(B.make_params(40, 64, block2d=1)) == 2
    assert _q(B.make_params(32, 64, block2d=1, rht=1)) == 5
    # 2D blocks packed for the transposed matrix only: row outputs are then not allowed
    assert _q(B.make_params(32, 64, layout=B.COLWISE, block2d=1), cr=P, sr=P, cc=P, sc=P) == 4
    # outputs for a layout that was not asked for
    assert _q(ok, cc=P, sc=P) == 4 and _q(ok, hc=P) == 4
    # columnwise requested but its outputs are missing
    assert _q(B.make_params(32, 64, layout=B.BOTH)) == 1
    # the transform with both orientations is refused
    assert _q(B.make_params(32, 64, layout=B.BOTH, rht=1), cc=P, sc=P) == 5
    # over-large shapes
    assert _q(B.make_params(1 << 32, 64)) == 2 and _q(B.make_params(1 << 30, 1 << 12)) == 2


def test_other_entry_points_validation_codes():
    ok = B.make_params(32, 64)
    assert B.tensor_scale_raw(P, ok, None, stream=0) == 1
    assert B.tensor_scale_raw(None, ok, P, stream=0) == 1
    assert B.tensor_scale_raw(P, B.make_params(32, 60), P, stream=0) == 2
    assert B.tensor_scale_raw(P + 4, ok, P, stream=0) == 3
    assert B.tensor_scale_raw(P, B.make_params(32, 64, layout=B.BOTH, rht=1), P, stream=0) == 5
    assert B.fake_quant_raw(P, ok, P, None, stream=0) == 1
    assert B.fake_quant_raw(P, B.make_params(32, 64, layout=B.BOTH), P, P, stream=0) == 4
    assert B.fake_quant_raw(P, ok, P, P + 6, stream=0) == 3
    assert B.dequantize_raw(None, P, P, 32, 64, B.ROWWISE, P, stream=0) == 1
    assert B.dequantize_raw(P, P, P, 32, 64, B.BOTH, P, stream=0) == 4
    assert B.dequantize_raw(P, P, P, 40, 64, B.BLOCK2D, P, stream=0) == 2
    assert B.dequantize_raw(P, P, P, 32, 40, B.ROWWISE, P, stream=0) == 2
    assert B.dequantize_raw(P, P, P, 24, 64, B.COLWISE, P, stream=0) == 2
    assert B.dequantize_raw(P, P + 3, P, 32, 64, B.ROWWISE, P, stream=0) == 3
    assert B.tensor_scale_ws_raw(P, ok, P, None, 4352, stream=0) == 1
    assert B.tensor_scale_ws_raw(P, ok, P, P, 4096, stream=0) == 4
    assert B.tensor_scale_ws_raw(P, ok, P, P + 4, 4352, stream=0) == 3
    assert B.tensor_scale_ws_raw(P, ok, None, P, 4352, stream=0) == 1
    L = B.lib()
    assert L.nvfp4_46_debug_e2m1_rtn_range(0, 16, None, None) == 1
    assert L.nvfp4_46_debug_e4m3_range(0, 0, C.c_void_p(P), None) == 2


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setenv("NVFP4_46_LIB", str(tmp_path / "nope.so"))
    monkeypatch.setattr(B, "_lib", None)
    with pytest.raises(FileNotFoundError):
        B.lib()


def test_every_hip_source_is_part_of_the_build():
    from pathlib import Path
    from paper_2512_02010_amd import build
    sources = {p.name for p in (Path(build.PKG) / "csrc").glob("*.hip")}
    assert sources == {Path(u[0]).name for u in build.UNITS}
    # each part number of a source compiled in parts appears exactly once
    for name in ("nvfp4_46.hip", "gemm.hip"):
        parts = sorted(list(u[1].values())[0] for u in build.UNITS if Path(u[0]).name == name)
        assert parts == list(range(7)), (name, parts)
