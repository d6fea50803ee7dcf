"""CPU: the oracle under AddressSanitizer and UndefinedBehaviorSanitizer.

`oracle_sanitizer_driver.c` includes the oracle's source and calls every entry point (all
layouts, rounding modes, selection rules, the Hadamard transform, fp32 input, 16x16 tiles, the
matrix product, the scalar codecs) on exactly-sized heap buffers; built with
-fsanitize=address,undefined -fno-sanitize-recover=all it exits non-zero on the first
out-of-bounds access or undefined operation."""
import subprocess
from pathlib import Path

import pytest

HERE = Path(__file__).resolve().parent
FLAGS = ["-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
         "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]


def _build(out: Path, *extra):
    subprocess.run(["gcc", *FLAGS, *extra, str(HERE / "oracle_sanitizer_driver.c"), "-o", str(out), "-lm"],
                   check=True)
    return out


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = _build(tmp_path / "driver")
    runs = [subprocess.run([str(exe)], capture_output=True, text=True, timeout=300) for _ in range(2)]
    for r in runs:
        assert r.returncode == 0, r.stderr[-4000:]
        assert "oracle sanitizer driver: ok" in r.stdout
    assert runs[0].stdout == runs[1].stdout          # and deterministic


def test_the_sanitizer_build_does_catch_an_out_of_bounds_store(tmp_path):
    # the same driver with one output buffer a byte short: the oracle's own store must trip it
    exe = _build(tmp_path / "driver_short", "-DPLANT_SHORT_BUFFER")
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300)
    assert r.returncode != 0
    assert "heap-buffer-overflow" in r.stderr
