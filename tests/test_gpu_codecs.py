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


def _words(k: np.ndarray, rng) -> torch.Tensor:
    """Random words whose top 24 bits are k (the low byte is noise nothing may depend on)."""
    w = (k.astype(np.uint32) << np.uint32(8)) | rng.integers(0, 256, k.size, dtype=np.uint32)
    return torch.from_numpy(w.view(np.int32)).cuda()


def test_e2m1_sr_matches_oracle():
    rng = np.random.default_rng(31)
    y = np.concatenate([rng.uniform(-7, 7, 30000), rng.standard_normal(10000) * 0.3,
                        [0.0, -0.0, 0.25, 0.5, 1.25, 5.5, 6.0, 6.5, -6.5, 1e-30, -1e-30, 1e30]])
    y = y.astype(np.float32)
    k = rng.integers(0, 1 << 24, y.size)
    # exact-threshold cases: u == p must not round up
    y[:3] = [1.25, 2.25, 5.5]
    k[:3] = [1 << 23, 1 << 22, 3 << 22]
    u = k.astype(np.float32) * np.float32(2.0 ** -24)
    got, fast = B.nvfp4_46_debug_e2m1_sr(torch.from_numpy(y).cuda(), _words(k, rng))
    got, fast = got.cpu().numpy(), fast.cpu().numpy()
    want = ref.e2m1_sr_n(y, u)
    assert np.array_equal(got, want)
    trusted = (fast & 0x80) == 0
    assert np.array_equal(fast[trusted], want[trusted]) and trusted.mean() > 0.999


def test_e2m1_sr_by_conversion_instruction_random_pairs_and_thresholds():
    """32 M random (y, word) pairs, half of them with the uniform placed within a few units of
    the threshold p = (|y| - lo) / (hi - lo): every code the kernels would keep is the oracle's,
    from 1 up the instruction's code is the oracle's always, and the kernels keep nearly all."""
    rng = np.random.default_rng(34)
    n = 1 << 24
    for part in range(2):
        mag = np.where(rng.random(n) < 0.5, rng.uniform(0.0, 7.0, n), 2.0 ** rng.uniform(-30.0, 3.0, n))
        y = (mag * rng.choice([-1.0, 1.0], n)).astype(np.float32)
        k = rng.integers(0, 1 << 24, n)
        if part == 1:
            a = np.minimum(np.abs(y), np.float32(6.0)).astype(np.float64)
            step = np.where(a < 2.0, 0.5, np.where(a < 4.0, 1.0, 2.0))
            p = a / step - np.floor(a / step)
            k = np.clip(np.floor(p * 2.0 ** 24).astype(np.int64) + rng.integers(-32, 33, n), 0, (1 << 24) - 1)
        u = k.astype(np.float32) * np.float32(2.0 ** -24)
        got, fast = B.nvfp4_46_debug_e2m1_sr(torch.from_numpy(y).cuda(), _words(k, rng))
        got, fast = got.cpu().numpy(), fast.cpu().numpy()
        want = ref.e2m1_sr_n(y, u)
        assert np.array_equal(got, want)
        trusted = (fast & 0x80) == 0
        code = fast & 0x0F
        assert np.array_equal(code[trusted], want[trusted])
        big = np.abs(y) >= 1.0
        assert np.array_equal(code[big], want[big])
        _log(f"part {part}: trusted {trusted.mean():.6f}, instruction differs on {int((code != want).sum())}")
        assert trusted.mean() > (0.999 if part == 0 else 0.5)
        if part == 1:
            assert (code != want).sum() > 1000      # the threshold cases do reach the difference


@pytest.mark.parametrize("sign", [0, 0x80000000])
def test_e2m1_sr_by_conversion_instruction_every_fp32(sign):
    """The stochastic-rounding conversion instruction as the kernels use it (value in the first
    source position, complemented random word), for every fp32 value up to infinity and several
    random words: wherever the kernels keep its code, that code is the oracle's; from 1 up it is
    the oracle's always; below 1 it is what the kernels' risk test assumes it to be (with
    P = floor(|y| 2^23): the lower grid point P >> 22, one step up iff (k >> 2) < P mod 2^22)."""
    rng = np.random.default_rng(33)
    inf, one, eight = f32_bits(float("inf")), f32_bits(1.0), f32_bits(8.0)
    ks = [0, (1 << 24) - 1, 1, 0x800000, 0x555555, int(rng.integers(0, 1 << 24))]
    flagged = 0
    for ik, k in enumerate(ks):
        u = float(np.float32(k) * np.float32(2.0 ** -24))
        word = ((k << 8) | 0x5A) - ((1 << 32) if k >= (1 << 23) else 0)
        pos = 0
        last = inf if ik == 0 else eight      # from 8 up every value saturates: one word is enough
        while pos <= last:
            n = min(CHUNK, last - pos + 1)
            _log(f"sr k=0x{k:06x} sign={sign >> 31}: bits 0x{pos:08x} .. +{n}")
            bits = torch.arange(pos, pos + n, dtype=torch.int64, device="cuda")
            sbits = bits + sign
            y = torch.where(sbits >= 2 ** 31, sbits - 2 ** 32, sbits).to(torch.int32).view(torch.float32)
            words = torch.full((n,), word, dtype=torch.int32, device="cuda")
            _, fast = B.nvfp4_46_debug_e2m1_sr(y, words)
            want = torch.from_numpy(ref.e2m1_sr_bits_range(pos + sign, n, u)).cuda()
            code, risk = fast & 0x0F, (fast & 0x80) != 0
            assert not bool((fast & 0x70).any())
            keep = ~risk | (bits >= one)           # 1 and above: always the oracle's
            bad = torch.nonzero(keep & (code != want)).flatten()[:5].cpu().numpy()
            assert bad.size == 0, (hex(k), [hex(pos + sign + int(i)) for i in bad])
            assert torch.equal(code & 8, torch.full_like(code, 8 if sign else 0))
            if pos < one:                          # below 1: the assumed form, flagged or not
                m = min(n, one - pos)
                P = torch.floor(y[:m].abs().to(torch.float64) * 2.0 ** 23).to(torch.int64)
                model = (P >> 22) + ((P & 0x3FFFFF) > (k >> 2)).to(torch.int64)
                assert torch.equal((code[:m] & 7).to(torch.int64), model)
            if k >= 16:
                flagged += int(risk.sum())
            del bits, sbits, y, words, fast, want, code, risk, keep
            pos += n
    # the risk test fires on a sliver only (|y| 2^25 within 4 of k; for k < 16 that sliver is
    # every value below about 2^-23 and is not counted)
    _log(f"flagged {flagged}")
    assert flagged < len(ks) * 64


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
