"""The two fixed operation orders the oracle had to choose (the paper states neither): the tree in
which a block's sixteen squared errors are added, and the stage order of the 16-point Hadamard
butterflies.  Each is written here a second time, as whole-array numpy fp32 operations rather
than the oracle's scalar loops, and compared bit for bit on inputs where the order matters; the
same inputs are shown to tell other orders apart, so the comparison is not vacuous.  This pins
the oracle to its stated reading of the order, not to the paper (which has no such statement).
"""
import numpy as np

from oracle import ref

F = np.float32


def _bits(a):
    return np.asarray(a, dtype=F).view(np.uint32)


def _tree_of_halves(e):
    """Each half 8 -> 4 -> 2 -> 1 by adding the upper to the lower part, then the two halves."""
    e = np.asarray(e, dtype=F).reshape(2, 8)
    a = e[:, :4] + e[:, 4:]
    b = a[:, :2] + a[:, 2:]
    c = b[:, 0] + b[:, 1]
    return F(c[0] + c[1])


def _sequential(e):
    s = F(0)
    for t in np.asarray(e, dtype=F):
        s = F(s + t)
    return s


def _adjacent_pairs(e):
    e = np.asarray(e, dtype=F)
    while e.size > 1:
        e = e[0::2] + e[1::2]
    return F(e[0])


def test_squared_errors_are_added_in_the_stated_tree():
    rng = np.random.default_rng(4690)
    differs_seq = differs_adj = 0
    for trial in range(400):
        v = (rng.standard_normal(16) * np.exp(rng.standard_normal(16))).astype(F)
        alpha = F(np.abs(v).max() / F(1536.0))
        for M in (6.0, 4.0):
            S = ref.block_scale(float(np.abs(v).max()), float(alpha), M)
            E, _, D = ref.block_with_scale(v, float(alpha), S)
            d = D.astype(F) - v              # one fp32 subtraction per element
            e = d * d                        # one fp32 multiplication per element
            assert _bits(E) == _bits(_tree_of_halves(e)), (trial, M)
            differs_seq += _bits(_sequential(e)) != _bits(E)
            differs_adj += _bits(_adjacent_pairs(e)) != _bits(E)
    # the inputs do distinguish this tree from the two other natural orders
    assert differs_seq > 100 and differs_adj > 100, (differs_seq, differs_adj)


def test_absolute_errors_use_the_same_tree():
    rng = np.random.default_rng(4691)
    for trial in range(200):
        v = rng.standard_normal(16).astype(F)
        D = (v + rng.standard_normal(16).astype(F) * F(0.1)).astype(F)
        want = _tree_of_halves(np.abs(D - v))
        assert _bits(ref.block_abs_metric(v, D, ref.SEL_46_MAE)) == _bits(want), trial


def _butterflies(v, strides):
    v = np.asarray(v, dtype=F).copy()
    for h in strides:
        g = v.reshape(16 // (2 * h), 2, h)
        top, bottom = g[:, 0, :].copy(), g[:, 1, :].copy()
        g[:, 0, :] = top + bottom
        g[:, 1, :] = top - bottom
        v = g.reshape(16)
    return v * F(0.25)


def test_hadamard_stages_run_from_stride_one_up():
    rng = np.random.default_rng(4692)
    differs_reversed = 0
    for trial in range(400):
        v = (rng.standard_normal(16) * np.exp(2 * rng.standard_normal(16))).astype(F)
        word = int(rng.integers(0, 1 << 16))
        signed = np.where((word >> np.arange(16)) & 1, -v, v).astype(F)
        got = ref.rht16(v, word)
        assert np.array_equal(_bits(got), _bits(_butterflies(signed, (1, 2, 4, 8)))), trial
        differs_reversed += not np.array_equal(_bits(got), _bits(_butterflies(signed, (8, 4, 2, 1))))
    assert differs_reversed > 100, differs_reversed


def _tile_errors(t, alpha, S, tree):
    rowerr = np.array([ref.block_with_scale(t[r], alpha, S)[0] for r in range(16)], dtype=F)
    return rowerr, tree(rowerr)


def test_tile_errors_are_the_row_errors_in_the_same_tree():
    """16x16 tiles (fp32 input): one element of a tile is moved, one fp32 step at a time, through
    a point where the two candidates' tile errors cross; around the crossing the oracle's
    choice must be `tree(row errors of 4) < tree(row errors of 6)` at every step, and adding
    the sixteen row errors one after the other would choose differently at some of them."""
    rng = np.random.default_rng(4693)
    crossings = steps_checked = sequential_differs = 0
    for trial in range(500):
        # magnitudes U^2.2: the distribution on which a tile's two candidates come out about even
        t = (np.sign(rng.standard_normal((16, 16))) * rng.random((16, 16)) ** 2.2).astype(F)
        alpha = ref.tensor_scale(t)
        b = float(np.abs(t).max())
        S6, S4 = ref.block_scale(b, alpha, 6.0), ref.block_scale(b, alpha, 4.0)
        err6, _ = _tile_errors(t, alpha, S6, _tree_of_halves)
        err4, _ = _tile_errors(t, alpha, S4, _tree_of_halves)

        def at(r, c, pattern):
            """Row errors, their difference and (r, c)'s two dequantized values with the
            element at (r, c) set to the fp32 value of this bit pattern."""
            row = t[r].copy()
            row[c] = np.uint32(pattern).view(F)
            e6, e4 = err6.copy(), err4.copy()
            e6[r], _, d6 = ref.block_with_scale(row, alpha, S6)
            e4[r], _, d4 = ref.block_with_scale(row, alpha, S4)
            gap = float(_tree_of_halves(e4)) - float(_tree_of_halves(e6))
            return e6, e4, gap, (float(d6[c]), float(d4[c]))

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
                _, _, g, dq = at(r, c, pattern)
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
        g_lo = at(r, c, lo)[2]
        while hi - lo > 1:
            mid = (lo + hi) // 2
            g = at(r, c, mid)[2]
            if g != 0 and (g < 0) == (g_lo < 0):
                lo = mid
            else:
                hi = mid
        crossings += 1
        for pattern in range(lo - 3, lo + 5):
            e6, e4, _, _ = at(r, c, pattern)
            tile = t.copy()
            tile[r, c] = np.uint32(pattern).view(F)
            assert ref.tensor_scale(tile) == alpha
            choice = int(ref.quantize_2d(tile, alpha)[2][0, 0])
            assert choice == int(_tree_of_halves(e4) < _tree_of_halves(e6)), (trial, pattern)
            sequential_differs += choice != int(_sequential(e4) < _sequential(e6))
            steps_checked += 1
    assert crossings >= 20 and sequential_differs >= 5, (crossings, steps_checked, sequential_differs)
