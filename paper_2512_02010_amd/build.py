"""Compile the HIP library in-tree: ``paper_2512_02010_amd/libnvfp4_46.so`` (gfx950 only)."""
from __future__ import annotations

import os
import shutil
import subprocess
from pathlib import Path

PKG = Path(__file__).resolve().parent
ROOT = PKG.parent
# (source, extra defines, object name).  Both sources are compiled in seven parts each, side
# by side: part 0 holds the entry points, parts 1..6 one group of kernels each (see the
# sources for the grouping).  The slowest parts come first so that they start first.
UNITS = [(PKG / "csrc" / "gemm.hip", {"NVFP4_46_GEMM_PART": part}, f"gemm.part{part}")
         for part in range(1, 5)]
UNITS += [(PKG / "csrc" / "nvfp4_46.hip", {"NVFP4_46_PART": part}, f"nvfp4_46.part{part}")
          for part in range(1, 7)]
UNITS += [(PKG / "csrc" / "gemm.hip", {"NVFP4_46_GEMM_PART": part}, f"gemm.part{part}")
          for part in (5, 6, 0)]
UNITS.append((PKG / "csrc" / "nvfp4_46.hip", {"NVFP4_46_PART": 0}, "nvfp4_46.part0"))
SO = PKG / "libnvfp4_46.so"

# -ffp-contract=off: the method's arithmetic is one rounding per operation.
# -packed-fp32-ops off: never let the compiler form v_pk_*_f32 from scalar float code.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unused-const-variable",
    # the copy instructions' inline assembly names m0 as clobbered; the compiler remarks that
    # m0 is a reserved register
    "-Wno-inline-asm",
]



def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and Path(cand).exists():
            return cand
    raise RuntimeError("hipcc not found")


def build(out: Path | None = None, defines: dict | None = None, extra: list | None = None) -> Path:
    """Compile every unit to an object (side by side) and link the shared library."""
    from concurrent.futures import ThreadPoolExecutor
    out = Path(out) if out else SO
    d = dict(defines or {})
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    common = [*flags, *(extra or []), f"-I{ROOT / 'include'}", f"-I{PKG / 'csrc'}"]
    objdir = PKG / "_build" / f"{out.stem}.{os.getpid()}"
    objdir.mkdir(parents=True, exist_ok=True)

    def compile_one(unit) -> Path:
        src, unit_defines, name = unit
        obj = objdir / (name + ".o")
        macros = [f"-D{k}={v}" for k, v in {**unit_defines, **d}.items()]
        subprocess.run([hipcc(), *common, *macros, "-c", str(src), "-o", str(obj)], check=True)
        return obj

    try:
        with ThreadPoolExecutor(min(len(UNITS), os.cpu_count() or 1)) as pool:
            objs = list(pool.map(compile_one, UNITS))
        tmp = out.with_suffix(f".tmp{os.getpid()}.so")
        subprocess.run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *map(str, objs),
                        "-o", str(tmp)], check=True)
        os.replace(tmp, out)
    finally:
        shutil.rmtree(objdir, ignore_errors=True)
    return out


if __name__ == "__main__":
    print(build())
