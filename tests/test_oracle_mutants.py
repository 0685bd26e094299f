"""Plant one mistake at a time in a copy of the oracle's C source (on the CPU) and check that
the pins notice: a dropped term, a wrong sign, index, rounding or constant must fail at
least one pin.  This is what makes the pins worth trusting as the oracle's anchor."""
import os
import subprocess

import pytest

import oracle
import pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "lpq_oracle.c")

# (name, text to find, replacement, how many occurrences must be replaced)
MUTANTS = [
    ("levels_2b_instead_of_2b_minus_1", "range / fqmax", "range / (fqmax + 1.0f)", 1),
    ("floor_instead_of_round", "float r = nearbyintf(t);\n                    int c = (r < 0.0f)", "float r = floorf(t);\n                    int c = (r < 0.0f)", 1),
    ("dequant_sign_of_zero", "volatile float v = p + z;", "volatile float v = p - z;", 1),
    ("quantize_ignores_zero", "lpq_oracle_h2f(wg[k]) - zf", "lpq_oracle_h2f(wg[k])", 1),
    ("matmul_reversed_k", "lpq_oracle_h2f(x[m * K + k])", "lpq_oracle_h2f(x[m * K + (K - 1 - k)])", 1),
    ("matmul_swapped_output_index", "y[m * N + n] = acc;", "y[(M - 1 - m) * N + n] = acc;", 1),
    ("nibble_order_sequential", "4 * (e / 2) + 16 * (e % 2)", "4 * e", 2),
    ("three_bit_fields_reversed", "16 * h + 3 * (P % 5)", "16 * h + 3 * (4 - P % 5)", 2),
    ("lane_uses_kq_major_rows", "*lane = 16 * ((kk % 32) / 8) + r;", "*lane = 4 * r + (kk % 32) / 8;", 1),
    ("rows_of_a_tile_consecutive", "t = (int)(n % 4), r = (int)((n % ORC_BLOCK_ROWS) / 4);", "t = (int)((n % ORC_BLOCK_ROWS) / 16), r = (int)(n % 16);", 1),
    ("tiles_ordered_by_tile_then_k", "(((size_t)block * (size_t)KT + (size_t)kt) * 4u + (size_t)t)", "(((size_t)block * 4u + (size_t)t) * (size_t)KT + (size_t)kt)", 1),
    ("scales_stored_row_major", "stored[g * N + n] = natural[n * G + g];", "stored[n * G + g] = natural[n * G + g];", 1),
    ("byte_order_of_8bit", "8 * (j % 2) + e]", "8 * (j % 2) + (7 - e)]", 2),
    ("fp16_pieces_per_lane_contiguous", "1024 * j + 16 * lane + 2 * e", "64 * lane + 16 * j + 2 * e", 4),
    ("sym_divides_by_128", "a / 127.0f", "a / 128.0f", 1),
    ("f2h_ties_away", "double r = nearbyint(q);", "double r = floor(q + 0.5);", 1),
    ("scale_from_max_only", "volatile float range = hi - lo;", "volatile float range = hi;", 1),
    ("dequant_wrong_group", "scales[n * G + k / ORC_GROUP]); z", "scales[n * G + (k / ORC_GROUP + 1) % G]); z", 1),
    ("bias_dropped", "if (bias) acc +=", "if (0) acc +=", 1),
    ("min_not_tracked", "if (v < lo) lo = v;", ";", 1),
    ("no_upper_clamp", "(r > fqmax ? qmax : (int)r)", "((int)r)", 1),
    ("sym_not_signed_on_unpack", "(int32_t)(int8_t)b", "(int32_t)b", 1),
    ("scale_kept_in_fp32_for_codes", "const float sf = lpq_oracle_h2f(sh), zf", "const float sf = s32, zf", 1),
]


@pytest.mark.parametrize("name,find,repl,count", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_planted_mistake(tmp_path, name, find, repl, count):
    text = open(SRC).read()
    assert text.count(find) == count, "mutation site moved: %r" % find
    c_path, so_path = tmp_path / "mutant.c", tmp_path / "mutant.so"
    c_path.write_text(text.replace(find, repl))
    subprocess.check_call(["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
                           "-Wno-unknown-pragmas", "-o", str(so_path), str(c_path), "-lm"])
    mutant = oracle.Oracle(str(so_path))
    caught = []
    for pin in pins.ALL_PINS:
        try:
            pin(mutant)
        except (AssertionError, ValueError):
            caught.append(pin.__name__)
            break
    assert caught, "no pin noticed the planted mistake %r" % name
