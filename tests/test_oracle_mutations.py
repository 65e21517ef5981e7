"""The pins of tests/test_oracle_pins.py must notice a plausible mistake in the oracle (CPU only).

Each case copies oracle/lora_oracle.c, plants one mistake in the copy by a textual edit (a
transposed operand, a dropped term, a wrong sign, an ignored index, an unstable sort, a wrong
rounding rule), builds it, lets the oracle's front end use it, and expects at least one pin
to fail.  The unedited copy must pass all of them.
"""
import ctypes as C
import os
import subprocess

import pytest

import test_oracle_pins as pins
from oracle import lora_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "lora_oracle.c")
GOLDEN = os.path.join(ROOT, "tests", "golden")

MUTATIONS = {
    "none": None,
    "A transposed": ("bf16_to_f64(A[(size_t)c * r + j])", "bf16_to_f64(A[(size_t)j * h_in + c])"),
    "B transposed": ("bf16_to_f64(B[(size_t)j * h_out + d])", "bf16_to_f64(B[(size_t)d * r + j])"),
    "scale dropped": ("double dl = s * acc;", "double dl = acc;"),
    "scale applied twice": ("double dl = s * acc;", "double dl = s * s * acc;"),
    "delta subtracted": ("if (y_out) y_out[o] = yi + dl;\n            if (y_bf16) y_bf16[o] = f64_to_bf16_rne(yi + dl);",
                         "if (y_out) y_out[o] = yi - dl;\n            if (y_bf16) y_bf16[o] = f64_to_bf16_rne(yi - dl);"),
    "src_row ignored": ("(src_row ? src_row[p] : p)", "(p)"),
    "expert ignored": ("const uint16_t *A = A_unit[(size_t)a * n_experts + e];",
                       "const uint16_t *A = A_unit[(size_t)a * n_experts];"),
    "expert and adapter swapped": ("const uint16_t *B = B_unit[(size_t)a * n_experts + e];",
                                   "const uint16_t *B = B_unit[((size_t)e * n_adapters + a) % ((size_t)n_adapters * n_experts)];"),
    "last input term dropped": ("for (int c = 0; c < h_in; ++c) {", "for (int c = 0; c + 1 < h_in; ++c) {"),
    "last rank term dropped": ("for (int j = 0; j < r; ++j) acc +=", "for (int j = 0; j + 1 < r; ++j) acc +="),
    "base output ignored": ("double yi = y_in ? bf16_to_f64(y_in[(size_t)p * ldy + d]) : 0.0;", "double yi = 0.0;"),
    "rows without adapter zeroed": ("if (y_bf16) y_bf16[o] = yb;", "if (y_bf16) y_bf16[o] = 0;"),
    "rounding truncates": ("double n = nearbyint(a / q);", "double n = floor(a / q);"),
    "rounding ties away": ("double n = nearbyint(a / q);", "double n = round(a / q);"),
    "sort unstable": ("for (int p = 0; p < P; ++p)\n        if (key[p] >= 0) perm[first[key[p]]++] = p;",
                      "for (int p = P - 1; p >= 0; --p)\n        if (key[p] >= 0) perm[first[key[p]]++] = p;"),
    "key order swapped": ("key[p] = (int64_t)a * n_experts + e;", "key[p] = (int64_t)e * n_adapters + a;"),
    "invalid ids kept": ("{ key[p] = -1; ++n_bad; continue; }", "{ key[p] = 0; ++n_bad; hist[0]++; continue; }"),
}


def run_pins():
    """Runs the pins with explicit arguments; returns the names of those that fail."""
    calls = [(pins.test_adapter_footprint_matches_paper, dict(golden_dir=GOLDEN)),
             (pins.test_hand_example, dict(golden_dir=GOLDEN))]
    calls += [(pins.test_merged_weight_form, dict(seed=s)) for s in (0, 1, 2)]
    for f in (pins.test_zero_B_gives_zero_delta_and_identical_output, pins.test_rank1_closed_form,
              pins.test_single_adapter_is_a_plain_gemm, pins.test_linearity_in_scale_and_input,
              pins.test_row_permutation_permutes_outputs_exactly,
              pins.test_rows_without_adapter_are_untouched, pins.test_out_of_range_ids_are_reported,
              pins.test_unit_selection_by_adapter_and_expert, pins.test_src_row_indirection,
              pins.test_tiny_exhaustive_exact_rational,
              pins.test_bf16_rounding_ties_to_even_and_matches_bit_trick,
              pins.test_y_bf16_is_single_rounding_of_the_exact_sum,
              pins.test_segments_invalid_ids_dropped_and_counted):
        calls.append((f, {}))
    calls += [(pins.test_segments_against_library_stable_sort, dict(seed=s, P=P, n=n, E=E))
              for s, P, n, E in [(2, 50, 4, 1), (3, 200, 7, 5), (5, 1000, 32, 8)]]
    failed = []
    for f, kw in calls:
        try:
            f(**kw)
        except AssertionError:
            failed.append(f.__name__)
    return failed


@pytest.mark.parametrize("name", list(MUTATIONS))
def test_pins_catch_a_planted_mistake(name, tmp_path, monkeypatch):
    text = open(SRC).read()
    if MUTATIONS[name] is not None:
        old, new = MUTATIONS[name]
        assert text.count(old) == 1, f"mutation site of '{name}' not found exactly once"
        text = text.replace(old, new)
    src = tmp_path / "oracle_mutant.c"
    lib = tmp_path / "liboracle_mutant.so"
    src.write_text(text)
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", str(lib),
                           str(src), "-lm"])
    O._load()                                        # the real one first, then swap
    monkeypatch.setattr(O, "_lib", O._declare(C.CDLL(str(lib))))
    failed = run_pins()
    if MUTATIONS[name] is None:
        assert failed == []
    else:
        assert failed, f"no pin noticed: {name}"
