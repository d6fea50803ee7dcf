"""Test helper: 16x16 fp32 tiles whose two candidates' tile errors are within a few fp32 steps of
a tie.  One element of a random tile is moved through a point where the difference of the two
tile errors changes sign while the element keeps its codes (a continuous crossing), found by
bisection on the element's bit pattern; the errors come from the oracle's per-row routine and
are added by the caller's `tree`.  Uses the oracle, so it lives with the tests."""
import numpy as np

from oracle import ref

F = np.float32

STEPS = (-512, -256, -128, -64, -16, -3, -2, -1, 0, 1, 2, 3, 4, 16, 64, 128, 256, 512)


def crossings(n_trials, seed, tree, alpha=None):
    """Yields (tile, r, c, first_pattern, alpha, S6, S4): setting tile[r, c] to the fp32 values of
    the bit patterns first_pattern + STEPS walks across the crossing (one fp32 step of the
    element moves a tile error by about 1/100 of its last bit, so the errors stay within a few
    last bits of each other, and exactly equal over long stretches, for hundreds of steps).  With
    alpha None every tile gets its own tensor scale (and keeps it while the element moves)."""
    rng = np.random.default_rng(seed)
    for trial in range(n_trials):
        # magnitudes U^2.2: the distribution on which a tile's two candidates come out about even
        t = (np.sign(rng.standard_normal((16, 16))) * rng.random((16, 16)) ** 2.2).astype(F)
        a = ref.tensor_scale(t) if alpha is None else alpha
        b = float(np.abs(t).max())
        S6, S4 = ref.block_scale(b, a, 6.0), ref.block_scale(b, a, 4.0)
        err6 = np.array([ref.block_with_scale(t[r], a, S6)[0] for r in range(16)], dtype=F)
        err4 = np.array([ref.block_with_scale(t[r], a, S4)[0] for r in range(16)], dtype=F)

        def at(r, c, pattern):
            row = t[r].copy()
            row[c] = np.uint32(pattern).view(F)
            e6, e4 = err6.copy(), err4.copy()
            e6[r], _, d6 = ref.block_with_scale(row, a, S6)
            e4[r], _, d4 = ref.block_with_scale(row, a, S4)
            return float(tree(e4)) - float(tree(e6)), (float(d6[c]), float(d4[c]))

        found = None
        for r, c in rng.integers(0, 16, (8, 2)):
            r, c = int(r), int(c)
            if not 0.02 * b < abs(t[r, c]) < 0.6 * b:      # not the maximum, not negligible
                continue
            # 48 samples over [v/2, 3v/2]; a sign change of the difference between two samples
            # that round to the same codes is a continuous crossing
            prev = None
            for k in range(48):
                pattern = int(F(t[r, c] * F(0.5 + k / 47.0)).view(np.uint32))
                g, dq = at(r, c, pattern)
                if prev and prev[2] == dq and g != 0 and prev[1] != 0 and (g < 0) != (prev[1] < 0):
                    found = (r, c, prev[0], pattern)
                    break
                prev = (pattern, g, dq)
            if found:
                break
        if not found:
            continue
        r, c, lo, hi = found
        if lo > hi:                      # a negative element: its patterns run the other way
            lo, hi = hi, lo
        g_lo = at(r, c, lo)[0]
        while hi - lo > 1:
            mid = (lo + hi) // 2
            g = at(r, c, mid)[0]
            if g != 0 and (g < 0) == (g_lo < 0):
                lo = mid
            else:
                hi = mid
        yield t, r, c, lo, a, S6, S4


BLOCK_STEPS = (-64, -16, -4, -3, -2, -1, 0, 1, 2, 3, 4, 5, 16, 64)


def block_crossings(n_trials, seed, tree, alpha, select=None, rounding=ref.RTN, uniforms=None,
                    samples=48, elements=8):
    """The same for one block of sixteen values under the tensor scale alpha: yields
    (block, i, first_pattern, S6, S4); block[i] set to the patterns first_pattern + BLOCK_STEPS
    walks across a crossing of the two candidates' block errors (here one fp32 step of the
    element moves an error by about one last bit, so the crossing is a few steps wide).
    `select` None: squared errors; ref.SEL_46_MAE: sums of absolute errors.  With stochastic
    rounding, `uniforms(k)` gives the sixteen uniforms of the k-th block yielded (they belong
    to its place in the caller's tensor); a failed search tries again for the same place."""
    rng = np.random.default_rng(seed)
    yielded = 0
    for trial in range(n_trials):
        v = (np.sign(rng.standard_normal(16)) * rng.random(16) ** 2.2).astype(F)
        v *= F(2.0) ** int(rng.integers(-8, 9))
        b = float(np.abs(v).max())
        S6, S4 = ref.block_scale(b, alpha, 6.0), ref.block_scale(b, alpha, 4.0)
        u = None if uniforms is None else uniforms(yielded)

        def at(i, pattern):
            w = v.copy()
            w[i] = np.uint32(pattern).view(F)
            E6, _, d6 = ref.block_with_scale(w, alpha, S6, rounding, u)
            E4, _, d4 = ref.block_with_scale(w, alpha, S4, rounding, u)
            if select is not None:
                E6, E4 = ref.block_abs_metric(w, d6, select), ref.block_abs_metric(w, d4, select)
            return float(E4) - float(E6), (float(d6[i]), float(d4[i]))

        found = None
        for i in rng.permutation(16)[:elements]:
            i = int(i)
            if not 0.02 * b < abs(v[i]) < 0.6 * b:
                continue
            prev = None
            for k in range(samples):
                pattern = int(F(v[i] * F(0.5 + k / (samples - 1.0))).view(np.uint32))
                g, dq = at(i, pattern)
                if prev and prev[2] == dq and g != 0 and prev[1] != 0 and (g < 0) != (prev[1] < 0):
                    found = (i, prev[0], pattern)
                    break
                prev = (pattern, g, dq)
            if found:
                break
        if not found:
            continue
        i, lo, hi = found
        if lo > hi:
            lo, hi = hi, lo
        g_lo = at(i, lo)[0]
        while hi - lo > 1:
            mid = (lo + hi) // 2
            g = at(i, mid)[0]
            if g != 0 and (g < 0) == (g_lo < 0):
                lo = mid
            else:
                hi = mid
        yielded += 1
        yield v, i, lo, S6, S4
