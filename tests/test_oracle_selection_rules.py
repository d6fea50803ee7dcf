"""Pins for the oracle's alternative 4-vs-6 selection rules (Section 3.1, Table 4):
mean absolute error and largest absolute error."""
from fractions import Fraction

import numpy as np

from oracle import ref
from paper_2512_02010_amd import workloads as wl
from tests._exact import E2M1_VALUES, e2m1_nearest, e4m3_value


def _rows(golden_dir):
    out = []
    for line in (golden_dir / "selection_rules_worked.txt").read_text().splitlines():
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        d = dict(tok.split("=", 1) for tok in line.split())
        for k in ("block", "D", "abs"):
            d[k] = [float(v) for v in d[k].split(",")]
        for k in ("M", "mae_sum", "absmax", "chosen_mae", "chosen_absmax"):
            d[k] = float(d[k])
        out.append(d)
    return out


def test_worked_blocks_under_mae_and_absmax(golden_dir):
    rows = _rows(golden_dir)
    assert len(rows) == 4
    for d in rows:
        x = d["block"]
        assert [abs(a - b) for a, b in zip(d["D"], x)] == d["abs"]
        assert sum(d["abs"]) == d["mae_sum"] and max(d["abs"]) == d["absmax"]
        key = "E6" if d["M"] == 6 else "E4"
        r_mae = ref.quantize_block(x, 1.0, select=ref.SEL_46_MAE)
        r_max = ref.quantize_block(x, 1.0, select=ref.SEL_46_ABSMAX)
        assert r_mae[key] == d["mae_sum"] and r_max[key] == d["absmax"]
        assert (4.0 if r_mae["four"] else 6.0) == d["chosen_mae"]
        assert (4.0 if r_max["four"] else 6.0) == d["chosen_absmax"]
        if d["M"] == d["chosen_mae"]:
            assert list(r_mae["D"][:4]) == d["D"]


def test_metrics_against_exact_rational():
    """On few-bit inputs with a power-of-two alpha every fp32 step is exact, so the
    metrics must equal their definitions evaluated in rational arithmetic."""
    rng = np.random.default_rng(41)
    n = 0
    for _ in range(300):
        v = (rng.integers(-48, 49, 16) * 0.25).astype(np.float32)
        alpha = float(2.0 ** rng.integers(-3, 2))
        for S in (0x30, 0x38, 0x40, 0x48):                  # power-of-two scales: exact reciprocals
            dec = e4m3_value(S) * Fraction(alpha)
            _, q, D = ref.block_with_scale(v, alpha, S)
            t = []
            for x in v:
                x = Fraction(float(x))
                code = e2m1_nearest(x / dec)
                mag = E2M1_VALUES[code & 7] * dec
                t.append(abs((-mag if code & 8 else mag) - x))
            assert Fraction(ref.block_abs_metric(v, D, ref.SEL_46_MAE)) == sum(t)
            assert Fraction(ref.block_abs_metric(v, D, ref.SEL_46_ABSMAX)) == max(t)
            n += 1
    assert n == 1200


def test_rules_select_by_their_own_metric_and_can_disagree():
    rng = np.random.default_rng(42)
    differ = {(a, b): 0 for a, b in ((0, 3), (0, 4), (3, 4))}
    for _ in range(1500):
        v = (rng.standard_normal(16) * np.exp(0.5 * rng.standard_normal(16))).astype(np.float32)
        alpha = float(np.float32(np.abs(v).max() * rng.uniform(1, 20)) / np.float32(1536.0))
        res = {}
        for sel in (ref.SEL_46_MSE, ref.SEL_46_MAE, ref.SEL_46_ABSMAX):
            r = ref.quantize_block(v, alpha, select=sel)
            r6 = ref.quantize_block(v, alpha, select=ref.SEL_FORCE6)
            r4 = ref.quantize_block(v, alpha, select=ref.SEL_FORCE4)
            if sel != ref.SEL_46_MSE:
                assert r["E6"] == ref.block_abs_metric(v, r6["D"], sel)
                assert r["E4"] == ref.block_abs_metric(v, r4["D"], sel)
                d6 = np.abs(r6["D"].astype(np.float64) - v)
                want = d6.sum() if sel == ref.SEL_46_MAE else d6.max()
                assert abs(r["E6"] - want) <= 1e-5 * max(want, 1e-30)
            assert r["four"] == int(r["E4"] < r["E6"])
            chosen = r4 if r["four"] else r6
            assert r["S"] == chosen["S"] and list(r["codes"]) == list(chosen["codes"])
            assert (r["E4"] if r["four"] else r["E6"]) <= r["E6"]
            res[sel] = r["four"]
        for a, b in differ:
            differ[(a, b)] += res[a] != res[b]
    assert all(c > 0 for c in differ.values()), differ      # the three rules are different rules


def test_tensor_entry_points_follow_the_rule():
    x = wl.bf16_bits(wl.make("c3", 64, 256))
    alpha = ref.tensor_scale(x)
    xf = (x.astype(np.uint32) << 16).view(np.float32)
    for sel in (ref.SEL_46_MAE, ref.SEL_46_ABSMAX):
        codes, scales, choice = ref.quantize(x, alpha, select=sel)
        E6, E4 = ref.block_errors(x, alpha, select=sel)
        assert np.array_equal(choice.astype(bool), E4 < E6)
        blk = ref.quantize_block(xf[5, 32:48], alpha, select=sel)
        assert scales[5, 2] == blk["S"] and choice[5, 2] == blk["four"]
        fq = ref.fake_quant(x, alpha, select=sel)
        assert np.array_equal(ref.dequantize(codes, scales, alpha, 64, 256), fq)
    c_mse = ref.quantize(x, alpha)[2]
    c_mae = ref.quantize(x, alpha, select=ref.SEL_46_MAE)[2]
    assert not np.array_equal(c_mse, c_mae)
