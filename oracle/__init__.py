"""Python face of the CPU oracle (spmm_oracle.c).

TEST INFRASTRUCTURE ONLY: the product path never imports this package.  Only
tests, the smoke check and the benchmark's cpu_baseline leg may use it.  It
imports nothing from the GPU package and shares no code with it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spmm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

OPS = {"sum": 0, "mean": 1, "max": 2, "min": 3}
STEP_FN = ctypes.CFUNCTYPE(ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_double)


def build(force: bool = False, src: str = _SRC, lib: str = _LIB) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over rows; no fast-math)."""
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(src):
        subprocess.run(["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-o", lib, src,
                        "-lm"], check=True)
    return lib


def _bind(path):
    L = ctypes.CDLL(path)
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    L.spmm_oracle.restype = ci
    L.spmm_oracle.argtypes = [i64, i64, i64, vp, vp, vp, vp, ci, vp, i64, vp, vp, ci]
    i32p = vp
    L.spmm_oracle_arg.restype = ci
    L.spmm_oracle_arg.argtypes = [i64, i64, i64, vp, vp, vp, vp, ci, vp, i64, vp, i32p, ci]
    L.spmm_oracle_transposed.restype = ci
    L.spmm_oracle_transposed.argtypes = [i64, i64, i64, vp, vp, vp, vp, ci, vp, vp, ci]
    L.spmm_oracle_pool_backward.restype = ci
    L.spmm_oracle_pool_backward.argtypes = [i64, i64, i64, vp, vp, vp, vp, vp, vp]
    L.spmm_oracle_csr_transpose.restype = ci
    L.spmm_oracle_csr_transpose.argtypes = [i64, i64, vp, vp, vp, ci, vp, vp, vp]
    L.spmm_oracle_custom.restype = ci
    L.spmm_oracle_custom.argtypes = [i64, i64, i64, vp, vp, vp, vp, ctypes.c_double, STEP_FN, vp]
    L.spmm_oracle_max_threads.restype = ci
    return L


def _load():
    global _lib
    if _lib is None:
        _lib = _bind(build())
    return _lib


def max_threads() -> int:
    return int(_load().spmm_oracle_max_threads())


def spmm(rowptr, colind, vals, B, op, rows=None, threads=0, _lib_override=None):
    """Reference result of C = A (x) B for CSR A.

    Returns (Cref, Sabs), both float64, shape (M, N) or (len(rows), N) when a row
    subset is given.  `vals` may be None (all stored values are 1).
    """
    L = _lib_override or _load()
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colind = np.ascontiguousarray(colind, dtype=np.int32)
    B = np.ascontiguousarray(B, dtype=np.float32)
    if vals is not None:
        vals = np.ascontiguousarray(vals, dtype=np.float32)
        assert vals.shape[0] == colind.shape[0]
    M = rowptr.shape[0] - 1
    K, N = B.shape
    assert int(rowptr[-1]) == colind.shape[0]
    if colind.size:
        assert colind.min() >= 0 and colind.max() < K
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        count = rows.shape[0]
        assert count == 0 or (rows.min() >= 0 and rows.max() < M)
    else:
        count = M
    Cref = np.empty((count, N), dtype=np.float64)
    Sabs = np.empty((count, N), dtype=np.float64)
    rc = L.spmm_oracle(M, K, N, rowptr.ctypes.data, colind.ctypes.data,
                       vals.ctypes.data if vals is not None else None, B.ctypes.data,
                       OPS[op] if isinstance(op, str) else int(op),
                       rows.ctypes.data if rows is not None else None, count,
                       Cref.ctypes.data, Sabs.ctypes.data, int(threads))
    if rc != 0:
        raise ValueError("spmm_oracle: bad argument")
    return Cref, Sabs


def _csr(rowptr, colind, vals):
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colind = np.ascontiguousarray(colind, dtype=np.int32)
    if vals is not None:
        vals = np.ascontiguousarray(vals, dtype=np.float32)
        assert vals.shape[0] == colind.shape[0]
    assert int(rowptr[-1]) == colind.shape[0]
    return rowptr, colind, vals


def spmm_arg(rowptr, colind, vals, B, op, rows=None, threads=0, _lib_override=None):
    """max / min and the position of the extreme: returns (Cref float64, arg int32); arg is the index
    into colind/vals of the first stored entry whose product, rounded once to fp32, has the bits of
    the result rounded once to fp32 (the position refers to the fp32 result the operator returns),
    -1 for empty rows."""
    L = _lib_override or _load()
    rowptr, colind, vals = _csr(rowptr, colind, vals)
    B = np.ascontiguousarray(B, dtype=np.float32)
    M, (K, N) = rowptr.shape[0] - 1, B.shape
    if colind.size:
        assert colind.min() >= 0 and colind.max() < K
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        count = rows.shape[0]
    else:
        count = M
    Cref = np.empty((count, N), dtype=np.float64)
    arg = np.empty((count, N), dtype=np.int32)
    rc = L.spmm_oracle_arg(M, K, N, rowptr.ctypes.data, colind.ctypes.data,
                           vals.ctypes.data if vals is not None else None, B.ctypes.data, OPS[op],
                           rows.ctypes.data if rows is not None else None, count,
                           Cref.ctypes.data, arg.ctypes.data, int(threads))
    if rc != 0:
        raise ValueError("spmm_oracle_arg: bad argument")
    return Cref, arg


def spmm_transposed(rowptr, colind, vals, dC, op, K, threads=0, _lib_override=None):
    """Gradient of sum / mean w.r.t. B: dB = A^T (x) dC from the CSR of A.  Returns (dBref, Sabs), K x N."""
    L = _lib_override or _load()
    rowptr, colind, vals = _csr(rowptr, colind, vals)
    dC = np.ascontiguousarray(dC, dtype=np.float32)
    M, N = dC.shape
    assert M == rowptr.shape[0] - 1
    if colind.size:
        assert colind.min() >= 0 and colind.max() < K
    dB = np.empty((K, N), dtype=np.float64)
    Sabs = np.empty((K, N), dtype=np.float64)
    rc = L.spmm_oracle_transposed(M, K, N, rowptr.ctypes.data, colind.ctypes.data,
                                  vals.ctypes.data if vals is not None else None, dC.ctypes.data,
                                  OPS[op], dB.ctypes.data, Sabs.ctypes.data, int(threads))
    if rc != 0:
        raise ValueError("spmm_oracle_transposed: bad argument")
    return dB, Sabs


def pool_backward(colind, vals, arg, dC, K, _lib_override=None):
    """Gradient of max / min w.r.t. B, routed through the positions `arg`.  Returns (dBref, Sabs)."""
    L = _lib_override or _load()
    colind = np.ascontiguousarray(colind, dtype=np.int32)
    if vals is not None:
        vals = np.ascontiguousarray(vals, dtype=np.float32)
    arg = np.ascontiguousarray(arg, dtype=np.int32)
    dC = np.ascontiguousarray(dC, dtype=np.float32)
    M, N = dC.shape
    assert arg.shape == (M, N) and (arg.size == 0 or (arg.min() >= -1 and arg.max() < colind.shape[0]))
    dB = np.empty((K, N), dtype=np.float64)
    Sabs = np.empty((K, N), dtype=np.float64)
    rc = L.spmm_oracle_pool_backward(M, K, N, colind.ctypes.data,
                                     vals.ctypes.data if vals is not None else None,
                                     arg.ctypes.data, dC.ctypes.data, dB.ctypes.data, Sabs.ctypes.data)
    if rc != 0:
        raise ValueError("spmm_oracle_pool_backward: bad argument")
    return dB, Sabs


def csr_transpose(rowptr, colind, vals, K, scale_by_row_length=False, _lib_override=None):
    """CSR of the transposed matrix (stable: rows of A in increasing order inside each result row).
    Returns (rowptrT int32[K+1], colindT int32[nnz], valsT float32[nnz])."""
    L = _lib_override or _load()
    rowptr, colind, vals = _csr(rowptr, colind, vals)
    M, nnz = rowptr.shape[0] - 1, colind.shape[0]
    if nnz:
        assert colind.min() >= 0 and colind.max() < K
    rowptrT = np.empty(K + 1, dtype=np.int32)
    colindT = np.empty(nnz, dtype=np.int32)
    valsT = np.empty(nnz, dtype=np.float32)
    rc = L.spmm_oracle_csr_transpose(M, K, rowptr.ctypes.data, colind.ctypes.data,
                                     vals.ctypes.data if vals is not None else None,
                                     int(bool(scale_by_row_length)), rowptrT.ctypes.data,
                                     colindT.ctypes.data, valsT.ctypes.data)
    if rc != 0:
        raise ValueError("spmm_oracle_csr_transpose: bad argument")
    return rowptrT, colindT, valsT


def spmm_custom(rowptr, colind, vals, B, init, step, _lib_override=None):
    """General SpMM-like operation: `init` is the initial accumulator, `step(acc, a, b)` a Python
    function folding one stored entry (a = stored value, b = B element), everything in double.
    Small inputs only (one interpreter call per product).  Returns Cref float64 (M, N)."""
    L = _lib_override or _load()
    rowptr, colind, vals = _csr(rowptr, colind, vals)
    B = np.ascontiguousarray(B, dtype=np.float32)
    M, (K, N) = rowptr.shape[0] - 1, B.shape
    if colind.size:
        assert colind.min() >= 0 and colind.max() < K
    Cref = np.empty((M, N), dtype=np.float64)
    rc = L.spmm_oracle_custom(M, K, N, rowptr.ctypes.data, colind.ctypes.data,
                              vals.ctypes.data if vals is not None else None, B.ctypes.data,
                              float(init), STEP_FN(step), Cref.ctypes.data)
    if rc != 0:
        raise ValueError("spmm_oracle_custom: bad argument")
    return Cref


def compare(op, C, Cref, Sabs):
    """Check a fp32 result against the oracle.

    sum / mean: |C - Cref| <= 1e-5 * Sabs + 1e-6 element-wise where the reference is finite; where
                the reference is +inf, -inf or NaN (non-finite inputs carried through Algorithm 1 in
                IEEE arithmetic) C must be that same infinity, or NaN for NaN.
    max / min : bit-for-bit equal to Cref rounded once to fp32.
    Returns (ok, worst) where worst is the largest error/bound ratio over the finite references
    (sum, mean) or the number of mismatching elements (max, min).
    """
    C = np.asarray(C)
    assert C.dtype == np.float32 and C.shape == Cref.shape
    if op in ("sum", "mean"):
        finite = np.isfinite(Cref)
        with np.errstate(invalid="ignore"):
            err = np.abs(C.astype(np.float64) - Cref)
            bound = 1e-5 * Sabs + 1e-6
            ratio = np.where(finite, err / bound, 0.0)
        ok = bool(np.all(np.isfinite(C[finite]))) and bool(np.all(err[finite] <= bound[finite]))
        same_special = (C[~finite] == Cref[~finite]) | (np.isnan(C[~finite]) & np.isnan(Cref[~finite]))
        ok = ok and bool(np.all(same_special))
        worst = float(ratio.max()) if ratio.size else 0.0
        return ok, worst
    want = Cref.astype(np.float32)
    bad = int(np.count_nonzero(C.view(np.uint32) != want.view(np.uint32)))
    return bad == 0, bad
