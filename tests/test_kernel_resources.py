"""CPU: register and scratch budgets of the kernels, read from the compiler's resource report.

hipcc cross-compiles for gfx950 without a GPU.  Two properties are pinned here because the
code silently depends on them:
  - the rowwise 4/6 kernel fits 64 vector registers (8 waves per SIMD) without spilling --
    the reason the rare undecided block is redone from memory instead of kept in registers;
  - the matrix-product kernels that wait for their asynchronous global -> LDS copies with
    hand-counted `s_waitcnt vmcnt(N)` use no scratch memory: a spill would add vector-memory
    instructions of the compiler's own and make those counts too small.
"""
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

from paper_2512_02010_amd import build


def _report(source: str, part_macro: str, part: int):
    flags = [f for f in build.HIPCC_FLAGS if f != "-shared"]
    r = subprocess.run([build.hipcc(), *flags, f"-I{build.ROOT / 'include'}", f"-I{build.PKG / 'csrc'}",
                        f"-D{part_macro}={part}", "-Rpass-analysis=kernel-resource-usage", "-c",
                        str(build.PKG / "csrc" / source), "-o", "/dev/null"],
                       capture_output=True, text=True, check=True)
    kernels, cur = {}, None
    for line in r.stderr.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            cur = kernels.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+(VGPRs|AGPRs|ScratchSize \[bytes/lane\]|Occupancy \[waves/SIMD\]): (\d+)", line)
        if m and cur is not None:
            cur[m.group(1).split(" ")[0]] = int(m.group(2))
    return kernels


def test_register_and_scratch_budgets():
    jobs = [("nvfp4_46.hip", "NVFP4_46_PART", 1), ("gemm.hip", "NVFP4_46_GEMM_PART", 5),
            ("gemm.hip", "NVFP4_46_GEMM_PART", 6)]
    with ThreadPoolExecutor(3) as pool:
        quant, dma, skinny = pool.map(lambda j: _report(*j), jobs)
    # k_flat<BF16 input, round to nearest, 4/6 by squared error, no transform, codes out>
    flat = [v for k, v in quant.items() if "6k_flatILb0ELi0ELi0ELb0ELi0E" in k]
    assert len(flat) == 1
    assert flat[0]["ScratchSize"] == 0 and flat[0]["VGPRs"] <= 64 and flat[0]["Occupancy"] == 8, flat[0]
    assert all(v["ScratchSize"] == 0 for v in quant.values())       # no quantizer kernel spills
    for kernels, name in ((dma, "k_gemm_dma"), (skinny, "k_gemm_skinny")):
        mine = {k: v for k, v in kernels.items() if name in k}
        assert len(mine) >= 2, (name, list(kernels))
        assert all(v["ScratchSize"] == 0 for v in mine.values()), mine
