"""Pins for the oracle's random numbers, stochastic rounding and Hadamard transform."""
import numpy as np

from oracle import ref
from tests._exact import philox4x32_10 as philox_py


def test_philox_known_answer_vectors(golden_dir):
    n = 0
    for line in (golden_dir / "philox4x32_10_kat.txt").read_text().splitlines():
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        w = [int(t, 16) for t in line.split()]
        assert len(w) == 10
        assert ref.philox4x32_10(w[0:4], w[4:6]) == tuple(w[6:10])
        n += 1
    assert n == 3


def test_philox_against_big_integer_twin():
    rng = np.random.default_rng(21)
    for _ in range(200):
        ctr = [int(v) for v in rng.integers(0, 1 << 32, 4)]
        key = [int(v) for v in rng.integers(0, 1 << 32, 2)]
        assert ref.philox4x32_10(ctr, key) == philox_py(ctr, key)


def test_sr_uniform_construction():
    seed = 0x0123456789ABCDEF
    for g in (0, 1, 2, 3, 4, 5, 1023, (1 << 32) + 7, (1 << 34) + 2, (1 << 40) - 1):
        q = g >> 2
        w = philox_py([q & 0xFFFFFFFF, q >> 32, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])
        want = (w[g & 3] >> 8) / float(1 << 24)
        assert ref.sr_uniform(seed, g) == want
        assert 0.0 <= want < 1.0
    us = np.array([ref.sr_uniform(77, g) for g in range(40000)])
    assert abs(us.mean() - 0.5) < 0.01 and abs(us.var() - 1 / 12) < 0.005
    hist = np.histogram(us, bins=16, range=(0, 1))[0]
    assert hist.min() > 2200 and hist.max() < 2800
    # different seeds / neighbouring elements decorrelate
    assert ref.sr_uniform(77, 10) != ref.sr_uniform(78, 10)


def test_rht_sign_word_construction():
    seed = 0xFEDCBA9876543210
    for B in (0, 1, 511, 1 << 33):
        w = philox_py([B & 0xFFFFFFFF, B >> 32, 0, 1], [seed & 0xFFFFFFFF, seed >> 32])
        assert ref.rht_sign_word(seed, B) == w[0]


def test_stochastic_rounding_is_unbiased_under_force6():
    """Mean over many uniforms of the SR-dequantized value tends to the input
    (standard NVFP4 + SR is unbiased, Appendix A.3)."""
    rng = np.random.default_rng(22)
    v = rng.standard_normal(16).astype(np.float32)
    v[3] = 2.9          # block maximum
    alpha = float(np.float32(5.0) / np.float32(1536.0))
    n = 4000
    acc = np.zeros(16)
    r_rtn = ref.quantize_block(v, alpha, ref.RTN, ref.SEL_FORCE6)
    dec = ref.e4m3_decode(r_rtn["S"]) * np.float32(alpha)
    for t in range(n):
        u = np.array([ref.sr_uniform(1000 + t, g) for g in range(16)], np.float32)
        r = ref.quantize_block(v, alpha, ref.SR, ref.SEL_FORCE6, u)
        assert r["S"] == r_rtn["S"]
        acc += r["D"]
    mean = acc / n
    # per-element standard error is at most step/2/sqrt(n) with step <= 2*dec;
    # an element whose scaled magnitude exceeds 6 (the block maximum, when its
    # scale was rounded down) saturates and is legitimately biased
    free = np.abs(v) <= 6 * float(dec)
    assert free.sum() >= 15
    assert np.all(np.abs(mean - v)[free] < 5 * float(dec) / np.sqrt(n) + 1e-7)


def test_sr_selection_uses_the_rounded_values():
    # "biased selection": the 4-vs-6 decision compares the errors of the two
    # stochastically rounded candidates, with the same u for both.
    rng = np.random.default_rng(23)
    flips = 0
    for _ in range(300):
        v = rng.standard_normal(16).astype(np.float32)
        alpha = float(np.float32(np.abs(v).max() * 2) / np.float32(1536.0))
        u = rng.random(16).astype(np.float32)
        r = ref.quantize_block(v, alpha, ref.SR, ref.SEL_46_MSE, u)
        b = float(np.abs(v).max())
        E6, q6, D6 = ref.block_with_scale(v, alpha, ref.block_scale(b, alpha, 6.0), ref.SR, u)
        E4, q4, D4 = ref.block_with_scale(v, alpha, ref.block_scale(b, alpha, 4.0), ref.SR, u)
        assert (r["E6"], r["E4"]) == (E6, E4)
        assert r["four"] == int(E4 < E6)
        assert list(r["codes"]) == list(q4 if r["four"] else q6)
        flips += r["four"] != ref.quantize_block(v, alpha)["four"]
    assert flips > 0      # SR does change some decisions relative to RTN


def _hadamard16():
    i = np.arange(16)
    pop = np.vectorize(lambda x: bin(x).count("1"))(i[:, None] & i[None, :])
    return np.where(pop % 2 == 0, 1.0, -1.0)


def test_rht_against_dense_matrix_fp64():
    rng = np.random.default_rng(24)
    H = _hadamard16()
    assert np.array_equal(H @ H, 16 * np.eye(16))
    for _ in range(200):
        v = (rng.standard_normal(16) * np.exp(rng.standard_normal(16))).astype(np.float32)
        w = int(rng.integers(0, 1 << 32))
        s = np.array([-1.0 if (w >> j) & 1 else 1.0 for j in range(16)])
        want = 0.25 * (H @ (s * v.astype(np.float64)))
        got = ref.rht16(v, w).astype(np.float64)
        assert np.allclose(got, want, rtol=0, atol=1e-6 * np.abs(v).max() * 4)
        # orthogonal: the norm is preserved
        assert abs(np.sum(got ** 2) - np.sum(v.astype(np.float64) ** 2)) < 1e-5 * np.sum(v.astype(np.float64) ** 2)


def test_rht_exact_on_small_integers_and_involution():
    rng = np.random.default_rng(25)
    H = _hadamard16()
    for _ in range(100):
        v = rng.integers(-64, 65, 16).astype(np.float32)
        once = ref.rht16(v, 0)
        assert np.array_equal(once.astype(np.float64), 0.25 * (H @ v.astype(np.float64)))
        # (H/4)(H/4) = I: applying it twice with unit signs gives the input back
        assert np.array_equal(ref.rht16(once, 0), v)
        # a sign word flips exactly the marked inputs before the butterflies
        w = int(rng.integers(0, 1 << 16))
        s = np.array([-1.0 if (w >> j) & 1 else 1.0 for j in range(16)], np.float32)
        assert np.array_equal(ref.rht16(v, w), ref.rht16(v * s, 0))
    # unit vectors give the rows of H/4; a constant block concentrates in element 0
    for j in range(16):
        e = np.zeros(16, np.float32)
        e[j] = 4.0
        assert np.array_equal(ref.rht16(e, 0), H[:, j].astype(np.float32))
    assert np.array_equal(ref.rht16(np.ones(16, np.float32), 0), np.eye(16, dtype=np.float32)[0] * 4)
