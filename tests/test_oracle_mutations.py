"""CPU: do the oracle's pins bite?  Single mistakes are planted in a copy of the oracle's
source (never in the oracle itself), each copy is built, and the pin test named beside the
mistake is run against it: it must fail.  A plausible slip anywhere in the oracle -- a dropped
term, a wrong sign or index, a swapped operand, a moved constant -- has to turn a test red.

Each entry: (what is planted, source text, replacement, the pin that must catch it).  The pin
named is the first one that fails in file order; most mistakes are caught by several.  One
candidate is left out because it changes nothing: without the clamp `if (a > 6) a = 6` in the
round-to-nearest routine, magnitudes above 6 still end at code 7 through the final lookup.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

from oracle import ref

ROOT = Path(__file__).resolve().parent.parent
SOURCE = ROOT / "oracle" / "nvfp4_46_ref.c"

MUTANTS = [
    ('ties go to 4 (<= for <)',
     'four = (E[1] < E[0]);',
     'four = (E[1] <= E[0]);',
     'tests/test_oracle_blocks.py::test_tie_keeps_six'),
    ('nibble order swapped',
     '(uint8_t)(q[i] | (q[i + 1] << 4))',
     '(uint8_t)(q[i+1] | (q[i] << 4))',
     'tests/test_oracle_fp32_input.py::test_fp32_tensor_equals_the_per_block_procedure_on_unrounded_values'),
    ('error term with the wrong sign',
     'float d = D[i] - v[i];',
     'float d = D[i] + v[i];',
     'tests/test_oracle_block2d.py::test_tile_selection_is_by_the_tile_error[0]'),
    ('a wrong index in the error tree',
     'for (int j = 0; j < 4; ++j) a[j] = p[j] + p[j + 4];',
     'for (int j = 0; j < 4; ++j) a[j] = p[j] + p[j + 3];',
     'tests/test_oracle_block2d.py::test_tile_selection_is_by_the_tile_error[0]'),
    ('error tree folds adjacent pairs instead of the upper onto the lower part',
     'for (int j = 0; j < 4; ++j) a[j] = p[j] + p[j + 4];',
     'for (int j = 0; j < 4; ++j) a[j] = p[2 * j] + p[2 * j + 1];',
     'tests/test_oracle_order_transcriptions.py::test_squared_errors_are_added_in_the_stated_tree'),
    ('Hadamard stages from stride eight down',
     'for (int h = 1; h < BLOCK; h <<= 1)\n    for (int i = 0; i < BLOCK; ++i)\n      if ((i & h) == 0) {',
     'for (int h = 8; h >= 1; h >>= 1)\n    for (int i = 0; i < BLOCK; ++i)\n      if ((i & h) == 0) {',
     'tests/test_oracle_order_transcriptions.py::test_hadamard_stages_run_from_stride_one_up'),
    ('tile error adds the row errors one after the other',
     'E[m] = error_sum(rowerr);',
     '{ float sum = 0.0f; for (int r = 0; r < BLOCK; ++r) sum += rowerr[r]; E[m] = sum; }',
     'tests/test_oracle_order_transcriptions.py::test_tile_errors_are_the_row_errors_in_the_same_tree'),
    ('both candidates scaled to 4',
     'S6 = ref_block_scale(b, alpha, 6.0f);',
     'S6 = ref_block_scale(b, alpha, 4.0f);',
     'tests/test_oracle_blocks.py::test_table3_worked_blocks'),
    ('E4M3 saturation threshold moved',
     'if (x >= 448.0f) return 0x7E;',
     'if (x >= 480.0f) return 0x7E;',
     'tests/test_oracle_blocks.py::test_block_scale_is_eq2_then_e4m3_cast'),
    ('E4M3 subnormal exponent off by one',
     'if (E < -6) E = -6;',
     'if (E < -7) E = -7;',
     'tests/test_oracle_blocks.py::test_block_scale_is_eq2_then_e4m3_cast'),
    ('Eq. (3) case boundary moved',
     'else if (a < 4.0f)',
     'else if (a < 3.0f)',
     'tests/test_oracle_blocks.py::test_table3_worked_blocks'),
    ('BF16 ties always round up',
     '(rest == 0x8000u && (keep & 1u))',
     '(rest == 0x8000u)',
     'tests/test_oracle_formats.py::test_bf16_conversions_match_torch'),
    ('Philox multiplier changed',
     '0xCD9E8D57u',
     '0xCD9E8D59u',
     'tests/test_oracle_random_rht.py::test_philox_known_answer_vectors'),
    ('uniform taken from the wrong Philox word',
     'w[g & 3] >> 8',
     'w[(g+1) & 3] >> 8',
     'tests/test_oracle_random_rht.py::test_sr_uniform_construction'),
    ('stochastic rounding compares with <=',
     'if (u < p) ++k;',
     'if (u <= p) ++k;',
     'tests/test_oracle_formats.py::test_e2m1_sr_bounds_and_probability'),
    ('first butterfly stage dropped',
     'for (int h = 1; h < BLOCK; h <<= 1)',
     'for (int h = 2; h < BLOCK; h <<= 1)',
     'tests/test_oracle_random_rht.py::test_rht_against_dense_matrix_fp64'),
    ('Hadamard scaled by 1/2',
     'v[j] *= 0.25f;',
     'v[j] *= 0.5f;',
     'tests/test_oracle_random_rht.py::test_rht_against_dense_matrix_fp64'),
    ('sign word from the wrong counter',
     '(uint32_t)(B >> 32), 0u, 1u}',
     '(uint32_t)(B >> 32), 0u, 0u}',
     'tests/test_oracle_random_rht.py::test_rht_sign_word_construction'),
    ('columnwise indices transposed',
     'int64_t c = (layout == REF_ROWWISE) ? blk * BLOCK + i : line;\n    g[i]',
     'int64_t c = (layout == REF_ROWWISE) ? blk * BLOCK + i : line;\n    if(layout!=REF_ROWWISE){int64_t t=r;r=c;c=t;}\n    g[i]',
     'tests/test_oracle_fp32_input.py::test_bf16_representable_values_give_the_bf16_results[0-0-2]'),
    ('Eq. (1) with 4 for 6',
     'amax / (6.0f * fp8_max)',
     'amax / (4.0f * fp8_max)',
     'tests/test_oracle_fp32_input.py::test_fp32_tensor_equals_the_per_block_procedure_on_unrounded_values'),
    ('dequantize drops the tensor scale',
     'float dec = ref_e4m3_decode(scales[line * NB + blk]) * alpha;',
     'float dec = ref_e4m3_decode(scales[line * NB + blk]);',
     'tests/test_oracle_fp32_input.py::test_fp32_tensor_equals_the_per_block_procedure_on_unrounded_values'),
    ('fp32 input rounded to BF16 on the way in',
     'return x.f32 ? ((const float *)x.p)[g] : ref_bf16_to_f32(((const uint16_t *)x.p)[g]);',
     'return x.f32 ? ref_bf16_to_f32(ref_f32_to_bf16(((const float *)x.p)[g])) : ref_bf16_to_f32(((const uint16_t *)x.p)[g]);',
     'tests/test_oracle_fp32_input.py::test_fp32_tensor_equals_the_per_block_procedure_on_unrounded_values'),
    ('matrix product: wrong scale index',
     'scales_b[lb * KB + k / BLOCK]',
     'scales_b[lb * KB + k / 8 % KB]',
     'tests/test_oracle_gemm.py::test_gemm_equals_float64_matmul_of_the_decoded_operands'),
    ('matrix product: nibbles of A swapped',
     'uint8_t ca = (k & 1) ? (ba >> 4) : (ba & 15)',
     'uint8_t ca = (k & 1) ? (ba & 15) : (ba >> 4)',
     'tests/test_oracle_gemm.py::test_gemm_equals_float64_matmul_of_the_decoded_operands'),
    ('matrix product: tensor scales added',
     'const double alpha = (double)alpha_a * (double)alpha_b;',
     'const double alpha = (double)alpha_a + (double)alpha_b;',
     'tests/test_oracle_gemm.py::test_gemm_equals_float64_matmul_of_the_decoded_operands'),
    ('matrix product: magnitude sum without |.|',
     'acc_abs += fabs(a * b);',
     'acc_abs += a * b;',
     'tests/test_oracle_gemm.py::test_gemm_equals_float64_matmul_of_the_decoded_operands'),
    ('matrix product: tile scale line off',
     'int64_t la = tiles_a ? m / BLOCK : m',
     'int64_t la = tiles_a ? m / 8 : m',
     'tests/test_oracle_gemm.py::test_gemm_with_tile_scales_equals_gemm_with_the_scales_repeated_per_row'),
    ('matrix product: output also written transposed',
     'C[m * N + n] = alpha * acc;',
     'C[(m * N + n)] = alpha * acc; if (m < N && n < M) C[n * N + m] = alpha * acc;',
     'tests/test_oracle_gemm.py::test_gemm_equals_float64_matmul_of_the_decoded_operands'),
    ('2D repacking: nibbles swapped',
     'codes_col[c * (rows / 2) + r / 2] = (uint8_t)(q0 | (q1 << 4));',
     'codes_col[c * (rows / 2) + r / 2] = (uint8_t)(q1 | (q0 << 4));',
     'tests/test_oracle_block2d.py::test_columnwise_packing_of_2d_blocks_is_the_transposed_matrix'),
    ('2D repacking: scales not transposed',
     'scales_col[tc * TR + tr] = scales[tr * TCB + tc];',
     'scales_col[tr * TCB + tc] = scales[tr * TCB + tc];',
     'tests/test_oracle_block2d.py::test_columnwise_packing_of_2d_blocks_is_the_transposed_matrix'),
    ('row slice: element index offset wrong',
     'ref_sr_uniform(sr_seed, g[i] + (uint64_t)x.row0 * (uint64_t)cols)',
     'ref_sr_uniform(sr_seed, g[i] + (uint64_t)x.row0)',
     'tests/test_oracle_tensor.py::test_quantizing_a_slice_of_rows_gives_that_slice_of_the_whole[1]'),
    ('row slice: sign-word position ignores the offset',
     ': x.row0 / BLOCK))));',
     ': 0))));',
     'tests/test_oracle_tensor.py::test_quantizing_a_slice_of_rows_gives_that_slice_of_the_whole[2]'),
    ('2D columnwise dequantize: scale index transposed',
     'scales_col[(c / BLOCK) * TR + r / BLOCK]',
     'scales_col[(r / BLOCK) * TR + c / BLOCK]',
     'tests/test_oracle_block2d.py::test_columnwise_packing_of_2d_blocks_is_the_transposed_matrix'),
]


def _pin_fails_on(mutant, workdir: Path):
    what, old, new, pin = mutant
    text = SOURCE.read_text()
    if text.count(old) < 1:
        return what, "the source text to replace was not found (update the table)"
    d = workdir / str(abs(hash((what, old))))
    d.mkdir()
    (d / "mutant.c").write_text(text.replace(old, new, 1))
    so = d / "mutant.so"
    r = subprocess.run(["gcc", *ref.CFLAGS, str(d / "mutant.c"), "-o", str(so), "-lm"],
                       capture_output=True, text=True)
    if r.returncode:
        return what, "the mutant does not compile: " + r.stderr[-300:]
    env = dict(os.environ, NVFP4_46_REF_LIB=str(so))
    r = subprocess.run([sys.executable, "-m", "pytest", pin, "-x", "-q", "-p", "no:cacheprovider"],
                       capture_output=True, text=True, env=env, cwd=str(ROOT))
    if r.returncode == 0:
        return what, f"NOT caught by {pin}"
    if " failed" not in r.stdout:
        return what, f"{pin} did not run to a failure: " + r.stdout[-300:]
    return what, None


def test_every_planted_mistake_turns_its_pin_red(tmp_path):
    assert len({m[0] for m in MUTANTS}) == len(MUTANTS) >= 30
    with ThreadPoolExecutor(min(8, os.cpu_count() or 1)) as pool:
        results = list(pool.map(lambda m: _pin_fails_on(m, tmp_path), MUTANTS))
    missed = [f"{what}: {why}" for what, why in results if why]
    assert not missed, "\n".join(missed)


def test_the_pins_pass_on_the_unchanged_source(tmp_path):
    # the same machinery with nothing planted: the copy must pass the pins the table names
    so = tmp_path / "same.so"
    subprocess.run(["gcc", *ref.CFLAGS, str(SOURCE), "-o", str(so), "-lm"], check=True)
    pins = sorted({m[3] for m in MUTANTS})
    r = subprocess.run([sys.executable, "-m", "pytest", *pins, "-q", "-p", "no:cacheprovider"],
                       capture_output=True, text=True, env=dict(os.environ, NVFP4_46_REF_LIB=str(so)),
                       cwd=str(ROOT))
    assert r.returncode == 0, r.stdout[-2000:]
