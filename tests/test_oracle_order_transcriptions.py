"""The two fixed operation orders the oracle had to choose (the paper states neither): the tree in
which a block's sixteen squared errors are added, and the stage order of the 16-point Hadamard
butterflies.  Each is written here a second time, as whole-array numpy fp32 operations rather
than the oracle's scalar loops, and compared bit for bit on inputs where the order matters; the
same inputs are shown to tell other orders apart, so the comparison is not vacuous.  This pins
the oracle to its stated reading of the order, not to the paper (which has no such statement).
"""
import numpy as np

from oracle import ref
from tests._near_ties import BLOCK_STEPS, STEPS, block_crossings, crossings

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


def test_tile_errors_are_the_row_errors_in_the_same_tree():
    """16x16 tiles (fp32 input): one element of a tile is moved, one fp32 step at a time, through
    a point where the two candidates' tile errors cross (tests/_near_ties.py); around the
    crossing the oracle's choice must be `tree(row errors of 4) < tree(row errors of 6)` at every
    step, and adding the sixteen row errors one after the other would choose differently at some
    of them."""
    n_crossings = steps_checked = sequential_differs = 0
    fours = []
    for t, r, c, first, alpha, S6, S4 in crossings(500, 4693, _tree_of_halves):
        n_crossings += 1
        for step in STEPS:
            pattern = first + step
            tile = t.copy()
            tile[r, c] = np.uint32(pattern).view(F)
            assert ref.tensor_scale(tile) == alpha
            e6 = np.array([ref.block_with_scale(tile[k], alpha, S6)[0] for k in range(16)], dtype=F)
            e4 = np.array([ref.block_with_scale(tile[k], alpha, S4)[0] for k in range(16)], dtype=F)
            choice = int(ref.quantize_2d(tile, alpha)[2][0, 0])
            assert choice == int(_tree_of_halves(e4) < _tree_of_halves(e6)), (r, c, pattern)
            sequential_differs += choice != int(_sequential(e4) < _sequential(e6))
            steps_checked += 1
            fours.append(choice)
    assert n_crossings >= 20 and sequential_differs >= 20, (n_crossings, steps_checked, sequential_differs)
    assert 0.25 < np.mean(fours) < 0.75, np.mean(fours)      # the steps do go both ways


def test_blocks_within_a_few_steps_of_a_tie_are_decided_by_the_stated_tree():
    """The same for 1x16 blocks: around a crossing of E4 and E6 the oracle's choice is the strict
    comparison of the two trees of squared errors, where sequential sums would differ."""
    alpha = float(F(1.0) / F(1536.0))
    n = sequential_differs = 0
    fours = []
    for v, i, first, S6, S4 in block_crossings(600, 4695, _tree_of_halves, alpha):
        n += 1
        for step in BLOCK_STEPS:
            w = v.copy()
            w[i] = np.uint32(first + step).view(F)
            e = {}
            for M, S in ((6, S6), (4, S4)):
                _, _, D = ref.block_with_scale(w, alpha, S)
                d = D.astype(F) - w
                e[M] = d * d
            got = ref.quantize_block(w, alpha)
            assert (got["S"], got["four"]) in ((S6, 0), (S4, 1))
            assert got["four"] == int(_tree_of_halves(e[4]) < _tree_of_halves(e[6])), (n, step)
            sequential_differs += got["four"] != int(_sequential(e[4]) < _sequential(e[6]))
            fours.append(got["four"])
    assert n >= 100 and sequential_differs >= 20, (n, sequential_differs)
    assert 0.25 < np.mean(fours) < 0.75, np.mean(fours)
