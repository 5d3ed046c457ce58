"""The pins must notice plausible mistakes in the oracle (CPU only).

Each case plants one mistake in a copy of the oracle's C source (a dropped
term, a wrong origin, a wrong sign, a wrong rounding ...), rebuilds it, and runs
the oracle's pin tests against the broken copy in a subprocess.  The pins pass
on the real source and must fail on every mutant.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "macko_oracle.c")
PIN_TESTS = ["tests/test_oracle_encoding.py", "tests/test_oracle_spmv.py", "tests/test_oracle_fp8.py"]

MUTANTS = {
    "first_delta_measured_from_column_0": ("int64_t prev = -1;", "int64_t prev = 0;"),
    "pads_one_entry_too_early": ("while (gap > D) {", "while (gap >= D) {"),
    "negative_zero_kept_as_nonzero": ("if ((w & 0x7FFFu) == 0) continue;      /* +0 and -0 are zeros */",
                                      "if (w == 0) continue;"),
    "padding_value_not_zero": ("values[e] = 0;\n        oracle_put_code(deltas, e, b_delta, (unsigned)(D - 1));",
                               "values[e] = 0x3C00;\n        oracle_put_code(deltas, e, b_delta, (unsigned)(D - 1));"),
    "nibble_order_swapped": ("return (deltas[bit >> 3] >> (bit & 7)) & ((1u << b) - 1u);",
                             "return (deltas[bit >> 3] >> ((bit & 7) ^ (b == 4 ? 4 : 0))) & ((1u << b) - 1u);"),
    "tail_granule_halved": ("return 128 / b_delta;", "return 64 / b_delta;"),
    "spmv_column_off_by_one": ("col += (int64_t)oracle_get_code(deltas, k, b_delta) + 1;\n      double p =",
                               "col += (int64_t)oracle_get_code(deltas, k, b_delta) + 1;\n      if (k == row_ptr[r]) col -= 1;\n      double p ="),
    "spmv_drops_last_entry_of_row": ("for (int64_t k = row_ptr[r]; k < row_ptr[r + 1]; ++k) {\n      col += (int64_t)oracle_get_code(deltas, k, b_delta) + 1;\n      double p =",
                                     "for (int64_t k = row_ptr[r]; k + 1 < row_ptr[r + 1]; ++k) {\n      col += (int64_t)oracle_get_code(deltas, k, b_delta) + 1;\n      double p ="),
    "abs_sum_keeps_sign": ("mag += fabs(p);\n    }\n    y64[r] = acc;\n    if (abs64) abs64[r] = mag;\n  }\n}\n\n/* ---- the product, by definition",
                           "mag += p;\n    }\n    y64[r] = acc;\n    if (abs64) abs64[r] = mag;\n  }\n}\n\n/* ---- the product, by definition"),
    "dense_product_skips_last_column": ("for (int64_t c = 0; c < C; ++c) {\n      double p =", "for (int64_t c = 0; c + 1 < C; ++c) {\n      double p ="),
    "subnormal_scale_wrong": ("v = ldexp((double)frac, -24);", "v = ldexp((double)frac, -25);"),
    "half_rounding_truncates": ("double q = nearbyint(ldexp(m, 11));", "double q = floor(ldexp(m, 11));"),
    "fp8_exponent_bias_off_by_one": ("v = ldexp((double)(frac + 8), exp - 10);", "v = ldexp((double)(frac + 8), exp - 9);"),
    "fp8_subnormal_scale_wrong": ("v = ldexp((double)frac, -9);", "v = ldexp((double)frac, -10);"),
    "fp8_top_binade_all_nan": ("else if (exp == 15 && frac == 7)   v = NAN;", "else if (exp == 15)   v = NAN;"),
    "fp8_negative_zero_kept_as_nonzero": ("if ((w & 0x7Fu) == 0) continue;          /* +0 and -0 are zeros */",
                                          "if (w == 0) continue;"),
    "fp8_count_and_fill_disagree_on_zero": ("if ((dense[r * ld + c] & 0x7Fu) == 0) continue;", "if (dense[r * ld + c] == 0) continue;"),
    "decoder_starts_at_column_0": ("int64_t col = -1;\n    for (int64_t k = row_ptr[r]; k < row_ptr[r + 1]; ++k) {\n      col += (int64_t)oracle_get_code(deltas, k, b_delta) + 1;\n      if (col >= C) return -(r + 1);",
                                   "int64_t col = 0;\n    for (int64_t k = row_ptr[r]; k < row_ptr[r + 1]; ++k) {\n      col += (int64_t)oracle_get_code(deltas, k, b_delta) + 1;\n      if (col >= C) return -(r + 1);"),
}


def run_pins(env_extra):
    env = dict(os.environ, **env_extra)
    return subprocess.run([sys.executable, "-m", "pytest", *PIN_TESTS, "-x", "-q", "-p", "no:cacheprovider"],
                          cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)


def test_pins_pass_on_an_unmodified_copy(tmp_path):
    copy = tmp_path / "oracle_copy.c"
    copy.write_text(open(SRC).read())
    r = run_pins({"MACKO_ORACLE_SRC": str(copy)})
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name", list(MUTANTS))
def test_pins_catch_mutant(name, tmp_path):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation site for {name} not found: the oracle source changed"
    mutant = tmp_path / f"{name}.c"
    mutant.write_text(text.replace(old, new))
    r = run_pins({"MACKO_ORACLE_SRC": str(mutant)})
    assert r.returncode != 0, f"no pin noticed the planted mistake '{name}'"
    assert "failed" in r.stdout or "error" in r.stdout.lower()
