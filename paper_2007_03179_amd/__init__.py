"""MI355X-native CSR SpMM / SpMM-like (sum, mean, max, min): HIP kernels behind a C ABI.

The kernels and the C entry points live in csrc/gespmm.hip (declared in include/gespmm.h);
this package only marshals arguments (binding.py) and builds the library (build.py).
"""
from .binding import (GespmmError, OPS, gespmm_custom_op_create, gespmm_custom_op_check, gespmm_custom_op_destroy, gespmm_csr_custom, gespmm_calibration_copy, gespmm_calibration_gather, gespmm_calibration_gather_shape, gespmm_csr, gespmm_csr_arg, gespmm_csr_b16,
                      gespmm_plan_b16, gespmm_csr_arg_b16, gespmm_csr_transpose_sorted, gespmm_csr_transpose_sorted_workspace_bytes,
                      gespmm_csr_simple, gespmm_csr_transpose, gespmm_csr_transpose_noalloc, gespmm_csr_transpose_workspace_bytes,
                      gespmm_csr_transposed, gespmm_plan, gespmm_pool_backward,
                      gespmm_csr_ex, gespmm_csr_arg_ex, gespmm_csr_workspace_bytes, gespmm_plan_ex,
                      gespmm_profiler_create, gespmm_profiler_finish, gespmm_tuning_t, make_tuning, gespmm_csr_prepared,
                      gespmm_status_string, gespmm_version, lib)

__all__ = ["GespmmError", "OPS", "gespmm_custom_op_create", "gespmm_custom_op_check", "gespmm_custom_op_destroy", "gespmm_csr_custom", "gespmm_calibration_copy", "gespmm_calibration_gather", "gespmm_calibration_gather_shape", "gespmm_csr", "gespmm_csr_arg", "gespmm_csr_b16",
           "gespmm_plan_b16", "gespmm_csr_arg_b16", "gespmm_csr_transpose_sorted", "gespmm_csr_transpose_sorted_workspace_bytes",
           "gespmm_csr_simple", "gespmm_csr_transpose", "gespmm_csr_transpose_noalloc", "gespmm_csr_transpose_workspace_bytes",
           "gespmm_csr_transposed", "gespmm_plan", "gespmm_pool_backward",
           "gespmm_csr_ex", "gespmm_csr_arg_ex", "gespmm_csr_workspace_bytes", "gespmm_plan_ex",
           "gespmm_profiler_create", "gespmm_profiler_finish", "gespmm_tuning_t", "make_tuning", "gespmm_csr_prepared",
           "gespmm_status_string", "gespmm_version", "lib"]
