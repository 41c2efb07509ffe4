"""Do the pins bite?  Each case below plants ONE plausible mistake in a copy of the oracle's source (on the
CPU, in a temporary directory), builds it, and runs the pin tests against that build in a child pytest: at
least one pin must fail for every mutant, and the unmodified copy must pass.  The mistakes are the ones a
wrong reading of the paper would produce: the sign<->bit map of the packing algorithm flipped, the row mean
of the dequantisation step dropped or applied to the wrong term, the element order inside a codeword or the
bit order inside an index reversed, a transposed output, an off-by-one index width, the ragged last chunk
read past the end of the row, the transform applied from the wrong side or with swapped Kronecker factors,
ties of the E-step broken the other way, a zero mean of the M-step sent to -1, an activation grid with one
level too many, ties or all fractions rounded the wrong way, the row offset left out."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "btc_oracle.cpp")

# (name, text in the oracle's source, replacement, pin files that must catch it)
MUTANTS = [
    ("sign_map_flipped", "const double sgn = ((pattern >> t) & 1u) ? 1.0 : -1.0;",
     "const double sgn = ((pattern >> t) & 1u) ? -1.0 : 1.0;", "test_oracle_pins.py"),
    ("row_mean_dropped", "W[r * in + k] = a * sgn + m;", "W[r * in + k] = a * sgn;", "test_oracle_pins.py"),
    ("row_mean_scaled_by_sign", "W[r * in + k] = a * sgn + m;", "W[r * in + k] = (a + m) * sgn;",
     "test_oracle_pins.py"),
    ("element_order_reversed", "const double sgn = ((pattern >> t) & 1u) ? 1.0 : -1.0;",
     "const double sgn = ((pattern >> (v - 1 - t)) & 1u) ? 1.0 : -1.0;", "test_oracle_pins.py"),
    ("index_bits_reversed_in_unpack", "code |= ((row[p >> 5] >> (p & 31)) & 1u) << q;\n      }\n      const uint32_t pattern",
     "code |= ((row[p >> 5] >> (p & 31)) & 1u) << (b - 1 - q);\n      }\n      const uint32_t pattern",
     "test_oracle_pins.py"),
    ("output_transposed", "Y[m * nrows + r] = acc;", "Y[r * M + m] = acc;", "test_oracle_pins.py"),
    ("index_width_floor", "while ((1L << b) < (long)K) ++b;", "while ((1L << (b + 1)) <= (long)K) ++b;",
     "test_oracle_pins.py"),
    ("last_chunk_not_cut", "if (k >= in) break;\n        const double sgn", "if (k >= in + 1) break;\n        const double sgn",
     "test_oracle_pins.py"),
    ("alpha_of_wrong_row", "const double a = (double)alpha[i];", "const double a = (double)alpha[r];",
     "test_oracle_pins.py"),
    ("words_msb_first", "if ((code >> q) & 1u) row[p >> 5] |= (1u << (p & 31));",
     "if ((code >> q) & 1u) row[p >> 5] |= (0x80000000u >> (p & 31));", "test_oracle_pins.py"),
    ("transform_from_the_left", "col[i] = sigma * ((double)P1[i1 * n1 + j1] * (double)P2[i2 * n2 + j2]);",
     "col[i] = sigma * ((double)P1[j1 * n1 + i1] * (double)P2[j2 * n2 + i2]);", "test_transform_pins.py"),
    ("kronecker_factors_swapped", "const long j1 = j / n2, j2 = j % n2;", "const long j1 = j % n1, j2 = j / n1;",
     "test_transform_pins.py"),
    ("transform_signs_dropped", "const double sigma = ((sign_bits[i >> 5] >> (i & 31)) & 1u) ? 1.0 : -1.0;",
     "const double sigma = 1.0;", "test_transform_pins.py"),
    ("estep_ties_to_highest", "if (best_k < 0 || d2 < best) {", "if (best_k < 0 || d2 <= best) {",
     "test_assign_pins.py"),
    ("estep_distance_not_squared", "d2 += (b - c) * (b - c);", "d2 += (b - c) > 0 ? (b - c) : (c - b);",
     "test_assign_pins.py"),
    ("mstep_zero_mean_to_minus", "if (sum[t] >= 0) c |= 1u << t;", "if (sum[t] > 0) c |= 1u << t;",
     "test_assign_pins.py"),
    ("quant_levels_power_of_two", "const float levels = (float)((1 << bits) - 1);", "const float levels = (float)(1 << bits);",
     "test_actquant_pins.py"),
    ("quant_rounds_half_up", "const float r = __builtin_nearbyintf(t / st);", "const float r = __builtin_floorf(t / st + 0.5f);",
     "test_actquant_pins.py"),
    ("quant_truncates", "const float r = __builtin_nearbyintf(t / st);", "const float r = __builtin_floorf(t / st);",
     "test_actquant_pins.py"),
    ("quant_symmetric_offset", "lo[m] = mn;", "lo[m] = 0.0f;", "test_actquant_pins.py"),
    ("quant_constant_row_step_zero", "const float st = range > 0.0f ? range / levels : 1.0f;",
     "const float st = range > 0.0f ? range / levels : 0.0f;", "test_actquant_pins.py"),
    ("groups_map_one_bit_per_weight", "const int g = (int)((grow[(2 * k) >> 5] >> ((2 * k) & 31)) & 3u);",
     "const int g = (int)((grow[k >> 5] >> (k & 31)) & 1u);", "test_groups_pins.py"),
    ("groups_mean_of_group_zero", "W[r * in + k] = (double)alpha[i * G + g] * sgn + (double)mu[i * G + g];",
     "W[r * in + k] = (double)alpha[i * G + g] * sgn + (double)mu[i * G];", "test_groups_pins.py"),
    ("groups_sign_map_flipped", "const double sgn = (pattern & (1u << t)) != 0u ? 1.0 : -1.0;",
     "const double sgn = (pattern & (1u << t)) != 0u ? -1.0 : 1.0;", "test_groups_pins.py"),
    ("groups_index_bits_reversed", "code += bit << q;", "code += bit << (b - 1 - q);", "test_groups_pins.py"),
    ("groups_parameters_transposed", "W[r * in + k] = (double)alpha[i * G + g] * sgn + (double)mu[i * G + g];",
     "W[r * in + k] = (double)alpha[g * out + i] * sgn + (double)mu[g * out + i];", "test_groups_pins.py"),
    ("mstep_empty_cluster_cleared", "if (size == 0) continue;", "if (size == 0) { codebook[k] = 0; continue; }",
     "test_assign_pins.py"),
]


def _run_pins(src_path, pin_file):
    env = dict(os.environ, BTC_ORACLE_SOURCE_UNDER_TEST=src_path)
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", pin_file), "-x", "-q",
                           "-m", "not gpu", "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True)


def test_unmodified_copy_passes_every_pin(tmp_path):
    src = tmp_path / "btc_oracle_copy.cpp"
    src.write_text(open(SRC).read())
    for pin_file in ("test_oracle_pins.py", "test_transform_pins.py", "test_assign_pins.py"):
        res = _run_pins(str(src), pin_file)
        assert res.returncode == 0, res.stdout[-2000:]


@pytest.mark.parametrize("name,old,new,pin_file", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_every_mutant_fails_a_pin(tmp_path, name, old, new, pin_file):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site of {name} not found exactly once"
    src = tmp_path / f"btc_oracle_{name}.cpp"
    src.write_text(text.replace(old, new))
    res = _run_pins(str(src), pin_file)
    assert res.returncode == 1, f"mutant {name} survived the pins (exit {res.returncode}):\n{res.stdout[-1500:]}"
    assert " failed" in res.stdout
