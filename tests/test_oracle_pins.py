"""The CPU oracle against its pins, and the pins against planted mistakes (CPU only)."""
import os
import re

import pytest

import oracle
from oracle_pins import GRAD_PINS, PINS

ORACLE_SRC = os.path.join(os.path.dirname(os.path.abspath(oracle.__file__)), "spmm_oracle.c")


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_oracle_passes_pin(pin):
    pin(oracle.spmm)


@pytest.mark.parametrize("pin", GRAD_PINS, ids=lambda p: p.__name__)
def test_gradient_side_oracle_passes_pin(pin):
    pin(oracle)


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
     "const int64_t row_end = rowptr[i + 1] - (rowptr[i + 1] - rowptr[i] > 2);", 0),
    # gradient-side functions
    ("arg_tie_goes_to_last", "if (where < 0 && same_bits32((float)x, target)) where = ptr;",
     "if (same_bits32((float)x, target)) where = ptr;"),
    ("arg_ties_on_exact_products", "if (where < 0 && same_bits32((float)x, target)) where = ptr;",
     "if (where < 0 && x == result && signbit(x) == signbit(result)) where = ptr;"),
    ("arg_value_from_the_wrong_fold", "result = (op == OP_MAX) ? fold_max(result, x) : fold_min(result, x);",
     "result = (op == OP_MAX) ? fold_min(result, x) : fold_max(result, x);"),
    ("arg_relative_to_row", "out_arg[j] = (int32_t)where;", "out_arg[j] = (int32_t)(where < 0 ? where : where - row_start);"),
    ("arg_zero_sign_ignored", "return ux.u == uy.u;", "return x == y;"),
    ("transposed_mean_multiplies", "if (op == OP_MEAN) w /= (double)len;", "if (op == OP_MEAN) w *= (double)len;"),
    ("transposed_not_transposed", "dBref[k * N + j] += x;", "dBref[(k < M ? i % K : k) * N + j] += x;", 0),
    ("transposed_sabs_signed", "Sabs[k * N + j] += fabs(x);", "Sabs[k * N + j] += x;", 0),
    ("pool_skips_entry_zero", "if (ptr < 0) continue;", "if (ptr <= 0) continue;"),
    ("pool_forgets_the_weight", "const double x = (vals ? (double)vals[ptr] : 1.0) * (double)dC[i * N + j];",
     "const double x = (double)dC[i * N + j];"),
    ("pool_adds_to_the_row_index", "dBref[k * N + j] += x;", "dBref[(i % K) * N + j] += x;", 1),
    ("transpose_prefix_sum_skipped", "rowptrT[k + 1] += rowptrT[k];", ";"),
    ("transpose_stores_column", "colindT[place] = (int32_t)i;", "colindT[place] = colind[ptr];"),
    ("transpose_scale_inverted", "if (scale_by_row_length) w /= len;", "if (scale_by_row_length) w *= len;"),
    ("transpose_places_not_advanced", "next[colind[ptr]]++;", "next[colind[ptr]];"),
    ("custom_restarts_every_step", "acc = step(acc, a, (double)B[(int64_t)colind[ptr] * N + j]);",
     "acc = step(init, a, (double)B[(int64_t)colind[ptr] * N + j]);"),
    ("custom_empty_row_keeps_init", "Cref[i * N + j] = rowptr[i + 1] > rowptr[i] ? acc : 0.0;", "Cref[i * N + j] = acc;"),
    ("arg_drop_last_term", "ptr < row_end; ++ptr", "ptr < row_end - 1; ++ptr", 1),
    ("arg_column_of_B_flipped", "B[k * N + j]", "B[k * N + (N - 1 - j)]", 1),
    ("arg_null_vals_as_zero", ": 1.0;", ": 0.0;", 1),
]
MUTANTS = [m if len(m) == 4 else (*m, None) for m in MUTANTS]


class _Mutant:
    """The oracle's Python face bound to a mutated library."""

    def __init__(self, lib):
        self.lib = lib

    def spmm(self, rowptr, colind, vals, B, op, rows=None):
        return oracle.spmm(rowptr, colind, vals, B, op, rows=rows, _lib_override=self.lib)

    def spmm_arg(self, rowptr, colind, vals, B, op, rows=None):
        return oracle.spmm_arg(rowptr, colind, vals, B, op, rows=rows, _lib_override=self.lib)

    def spmm_transposed(self, rowptr, colind, vals, dC, op, K):
        return oracle.spmm_transposed(rowptr, colind, vals, dC, op, K, _lib_override=self.lib)

    def pool_backward(self, colind, vals, arg, dC, K):
        return oracle.pool_backward(colind, vals, arg, dC, K, _lib_override=self.lib)

    def spmm_custom(self, rowptr, colind, vals, B, init, step):
        return oracle.spmm_custom(rowptr, colind, vals, B, init, step, _lib_override=self.lib)

    def csr_transpose(self, rowptr, colind, vals, K, scale_by_row_length=False):
        return oracle.csr_transpose(rowptr, colind, vals, K, scale_by_row_length, _lib_override=self.lib)


@pytest.mark.parametrize("name,old,new,which", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_reject_planted_mistake(tmp_path, name, old, new, which):
    src = open(ORACLE_SRC).read()
    which = which or 0                      # occurrence to change (0-based); the forward function comes first
    parts = src.split(old)
    assert len(parts) > which + 1, f"mutation site {which} for {name} not found"
    mutated_src = old.join(parts[: which + 1]) + new + old.join(parts[which + 1:])
    assert mutated_src != src
    mutated = tmp_path / f"oracle_{name}.c"
    mutated.write_text(mutated_src)
    m = _Mutant(oracle._bind(oracle.build(force=True, src=str(mutated), lib=str(tmp_path / f"lib_{name}.so"))))

    rejected = []
    for pin in PINS:
        try:
            pin(m.spmm)
        except AssertionError:
            rejected.append(pin.__name__)
    for pin in GRAD_PINS:
        try:
            pin(m)
        except AssertionError:
            rejected.append(pin.__name__)
    assert rejected, f"no pin noticed the planted mistake '{name}'"
