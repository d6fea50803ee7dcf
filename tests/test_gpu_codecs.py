"""GPU: the device codecs the kernels use, compared with the CPU oracle over their
whole input ranges (through the C-ABI debug entry points)."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2512_02010_amd import binding as B
from tests._exact import f32_bits

pytestmark = pytest.mark.gpu

CHUNK = 1 << 27


def _log(msg):
    print(msg, flush=True)


def test_decode_tables_match_oracle():
    t = B.nvfp4_46_debug_decode_tables().cpu().numpy()
    for c in range(16):
        want = np.float32(ref.e2m1_decode(c))
        assert t[c] == want and np.signbit(t[c]) == np.signbit(want), c
    for b in range(256):
        if (b & 0x7F) == 0x7F:
            continue
        assert t[16 + b] == np.float32(ref.e4m3_decode(b & 0x7F)), b


def _sweep(gpu_fn, ref_fn, first, last_inclusive, what):
    pos = first
    while pos <= last_inclusive:
        n = min(CHUNK, last_inclusive - pos + 1)
        _log(f"{what}: bits 0x{pos:08x} .. +{n}")
        got = gpu_fn(pos, n).cpu().numpy()
        want = ref_fn(pos, n)
        if not np.array_equal(got, want):
            bad = np.flatnonzero(got != want)[:5]
            raise AssertionError(
                f"{what}: first mismatches at bits {[hex(pos + int(i)) for i in bad]}: "
                f"gpu {got[bad]} oracle {want[bad]}")
        pos += n


def test_e2m1_rtn_every_finite_fp32():
    """Round-to-nearest-even onto E2M1, all finite inputs of both signs and +-inf."""
    inf = f32_bits(float("inf"))
    _sweep(B.nvfp4_46_debug_e2m1_rtn_range, ref.e2m1_rtn_bits_range, 0x00000000, inf, "e2m1 +")
    _sweep(B.nvfp4_46_debug_e2m1_rtn_range, ref.e2m1_rtn_bits_range, 0x80000000, 0x80000000 + inf,
           "e2m1 -")


def test_e4m3_encode_every_nonnegative_fp32():
    """Round-to-nearest-even onto E4M3 with saturation at 448, all inputs in [0, +inf]."""
    _sweep(B.nvfp4_46_debug_e4m3_range, ref.e4m3_encode_bits_range, 0x00000000,
           f32_bits(float("inf")), "e4m3")


def test_bf16_rounding():
    tops = [0x0000, 0x0001, 0x007F, 0x0080, 0x3F7F, 0x3F80, 0x3FFF, 0x4000, 0x42FE, 0x7F00, 0x7F7E,
            0x7F7F, 0x8000, 0x8080, 0xBF80, 0xC2FF, 0xFF7E, 0xFF7F]
    for top in tops:
        got = B.nvfp4_46_debug_bf16_range(top << 16, 1, 1 << 16).cpu().numpy().view(np.uint16)
        want = np.array([ref.f32_to_bf16(float(np.uint32((top << 16) + i).view(np.float32)))
                         for i in range(0, 1 << 16, 251)], dtype=np.uint16)
        assert np.array_equal(got[::251], want), hex(top)
        # exhaustive within the word by the rule itself: keep + (rest > half or tie & odd)
        rest = np.arange(1 << 16, dtype=np.uint32)
        exp = (top + ((rest > 0x8000) | ((rest == 0x8000) & ((top & 1) == 1)))).astype(np.uint16)
        assert np.array_equal(got, exp), hex(top)
    # a strided sweep over all finite values against the oracle
    n = 1 << 22
    stride = 1021
    bits = (np.arange(n, dtype=np.uint64) * stride).astype(np.uint32)
    got = B.nvfp4_46_debug_bf16_range(0, stride, n).cpu().numpy().view(np.uint16)
    finite = (bits & 0x7F800000) != 0x7F800000
    sample = np.flatnonzero(finite)[::97]
    want = np.array([ref.f32_to_bf16(float(bits[i:i + 1].view(np.float32)[0])) for i in sample],
                    dtype=np.uint16)
    assert np.array_equal(got[sample], want)


def test_e2m1_sr_matches_oracle():
    rng = np.random.default_rng(31)
    y = np.concatenate([rng.uniform(-7, 7, 30000), rng.standard_normal(10000) * 0.3,
                        [0.0, -0.0, 0.25, 0.5, 1.25, 5.5, 6.0, 6.5, -6.5, 1e-30, -1e-30, 1e30]])
    y = y.astype(np.float32)
    u = (rng.integers(0, 1 << 24, y.size).astype(np.float32) * np.float32(2.0 ** -24))
    # exact-threshold cases: u == p must not round up
    y[:3] = [1.25, 2.25, 5.5]
    u[:3] = [0.5, 0.25, 0.75]
    got = B.nvfp4_46_debug_e2m1_sr(torch.from_numpy(y).cuda(), torch.from_numpy(u).cuda())
    got = got.cpu().numpy()
    want = np.array([ref.e2m1_sr(float(a), float(b)) for a, b in zip(y, u)], dtype=np.uint8)
    assert np.array_equal(got, want)


def test_philox_matches_oracle_and_known_answers(golden_dir):
    rows = []
    for line in (golden_dir / "philox4x32_10_kat.txt").read_text().splitlines():
        line = line.strip()
        if line and not line.startswith("#"):
            rows.append([int(t, 16) for t in line.split()])
    for w in rows:
        ctr = torch.tensor([w[0:4]], dtype=torch.int64).to(torch.int32).cuda()
        out = B.nvfp4_46_debug_philox(ctr, w[4], w[5]).cpu().numpy().view(np.uint32)[0]
        assert [int(v) for v in out] == w[6:10]
    rng = np.random.default_rng(32)
    ctr = rng.integers(0, 1 << 32, (4096, 4), dtype=np.uint64).astype(np.uint32)
    k0, k1 = 0x9ABCDEF0, 0x12345678
    out = B.nvfp4_46_debug_philox(torch.from_numpy(ctr.view(np.int32)).cuda(), k0, k1)
    out = out.cpu().numpy().view(np.uint32)
    for i in range(0, 4096, 17):
        assert tuple(int(v) for v in out[i]) == ref.philox4x32_10([int(v) for v in ctr[i]], (k0, k1))
