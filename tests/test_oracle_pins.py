"""The CPU oracle against its pins, and the pins against planted mistakes (CPU only)."""
import os
import re

import pytest

import oracle
from oracle_pins import PINS

ORACLE_SRC = os.path.join(os.path.dirname(os.path.abspath(oracle.__file__)), "spmm_oracle.c")


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_oracle_passes_pin(pin):
    pin(oracle.spmm)


# One plausible single mistake each (dropped term, wrong sign, wrong index, flipped operand,
# wrong divisor, wrong initial value, ...).  All stay inside array bounds.
MUTANTS = [
    ("drop_last_term", "ptr < row_end; ++ptr", "ptr < row_end - 1; ++ptr"),
    ("skip_first_term", "ptr = row_start; ptr", "ptr = row_start + (row_end - row_start > 1); ptr"),
    ("wrong_sign", "else result += x;", "else result -= x;"),
    ("column_of_B_flipped", "B[k * N + j]", "B[k * N + (N - 1 - j)]"),
    ("colind_not_advanced", "colind[ptr]", "colind[row_start]"),
    ("val_not_advanced", "(double)vals[ptr]", "(double)vals[row_start]"),
    ("mean_divisor_off_by_one", "result /= (double)len;", "result /= (double)(len + 1);"),
    ("mean_bound_not_scaled", "sabs /= (double)len;", ";"),
    ("sabs_without_abs", "sabs += fabs(x);", "sabs += x;"),
    ("max_init_zero", "(op == OP_MAX) ? -INFINITY", "(op == OP_MAX) ? 0.0"),
    ("min_init_zero", "(op == OP_MIN) ? INFINITY", "(op == OP_MIN) ? 0.0"),
    ("max_compares_backwards", "if (x > acc) return x;", "if (x < acc) return x;"),
    ("min_is_max", "if (x < acc) return x;", "if (x > acc) return x;"),
    ("signed_zero_rule_max", "x == acc && !signbit(x)", "x == acc && signbit(x) && 0"),
    ("signed_zero_rule_min", "x == acc && signbit(x)) return x;", "x == acc && !signbit(x)) return x;"),
    ("null_vals_as_zero", ": 1.0;", ": 0.0;"),
    ("empty_row_not_zero", "if (len == 0) {", "if (len < 0) {"),
    ("product_rounded_to_fp32", "const double x = a * (double)B[k * N + j];",
     "const double x = (double)((float)a * B[k * N + j]);"),
    ("row_subset_ignored", "rows ? rows[r] : r;", "r;"),
    ("next_row_start_as_end", "const int64_t row_end = rowptr[i + 1];",
     "const int64_t row_end = rowptr[i + 1] - (rowptr[i + 1] - rowptr[i] > 2);"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_reject_planted_mistake(tmp_path, name, old, new):
    src = open(ORACLE_SRC).read()
    assert src.count(old) == 1, f"mutation site for {name} must occur exactly once"
    mutated = tmp_path / f"oracle_{name}.c"
    mutated.write_text(src.replace(old, new))
    lib = oracle._bind(oracle.build(force=True, src=str(mutated), lib=str(tmp_path / f"lib_{name}.so")))

    def mutant(rowptr, colind, vals, B, op, rows=None):
        return oracle.spmm(rowptr, colind, vals, B, op, rows=rows, _lib_override=lib)

    rejected = []
    for pin in PINS:
        try:
            pin(mutant)
        except AssertionError:
            rejected.append(pin.__name__)
    assert rejected, f"no pin noticed the planted mistake '{name}'"
