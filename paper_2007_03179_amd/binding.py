"""ctypes binding of libgespmm.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/gespmm.h).  Tensors
are torch CUDA tensors used purely as device memory; the stream is torch's current
stream unless one is given.  Nothing is computed on this side, and there is no
fallback: a missing library is an error.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgespmm.so")

OPS = {"sum": 0, "mean": 1, "max": 2, "min": 3}
GESPMM_OK = 0


class GespmmError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"gespmm status {status}: {text}")
        self.status = status


class gespmm_plan_t(ctypes.Structure):
    _fields_ = [("vec", ctypes.c_int32), ("lanes_per_row", ctypes.c_int32),
                ("tiles_per_lane", ctypes.c_int32), ("slots", ctypes.c_int32),
                ("chunk_nnz", ctypes.c_int32), ("col_blocks", ctypes.c_int32),
                ("chunks", ctypes.c_int64), ("grid_x", ctypes.c_int64),
                ("block_threads", ctypes.c_int32), ("xcd_remap", ctypes.c_int32),
                ("short_len", ctypes.c_int32), ("lds_bytes", ctypes.c_int32),
                ("k_parts", ctypes.c_int32), ("row_window", ctypes.c_int32), ("workspace_bytes", ctypes.c_int64)]


class gespmm_tuning_t(ctypes.Structure):
    _fields_ = [("lanes_per_row", ctypes.c_int32), ("tiles_per_lane", ctypes.c_int32),
                ("xcd_remap", ctypes.c_int32), ("chunk_nnz", ctypes.c_int32),
                ("short_len", ctypes.c_int32), ("k_parts", ctypes.c_int32), ("longest_row", ctypes.c_int32), ("wide_addresses", ctypes.c_int32)]


def _tuning(t):
    """None, a gespmm_tuning_t, a dict of field names, or up to eight numbers in field order (-1 = automatic)."""
    if t is None or isinstance(t, gespmm_tuning_t):
        return t
    out = gespmm_tuning_t(-1, -1, -1, -1, -1, -1, -1, -1)
    if isinstance(t, dict):
        for name, value in t.items():
            if name not in dict(gespmm_tuning_t._fields_):
                raise KeyError(name)
            setattr(out, name, int(value))
    else:
        for (name, _), value in zip(gespmm_tuning_t._fields_, t):
            setattr(out, name, int(value))
    return out


def make_tuning(t):
    """A gespmm_tuning_t built once from a dict of field names (or a sequence in field order), for callers that
    make many calls with the same overrides: passing the structure skips the conversion on every call."""
    return _tuning(t)


def _tuning_ref(t):
    t = _tuning(t)
    return None if t is None else ctypes.byref(t)


_lib = None


def lib():
    """The loaded library.  It is built by build.py; if it is not there it is compiled now (hipcc,
    gfx950), and if that is impossible this raises: there is no other code path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            try:
                from . import build as _build
                _build.build(force=True)
            except Exception as exc:
                raise FileNotFoundError(
                    f"{LIB_PATH} is missing and could not be compiled ({exc}): run "
                    "`python -c 'import __graft_entry__ as g; g.build()'`; there is no fallback path") from exc
        L = ctypes.CDLL(LIB_PATH)
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        L.gespmm_csr.restype = ci
        L.gespmm_csr.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, vp, ci, vp]
        L.gespmm_csr_b16.restype = ci
        L.gespmm_csr_b16.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, ci, vp, ci, vp]
        L.gespmm_csr_arg_b16.restype = ci
        L.gespmm_csr_arg_b16.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, ci, vp, vp, ci, vp]
        L.gespmm_plan_b16.restype = ci
        L.gespmm_plan_b16.argtypes = [i64, i64, i64, ci, ci, ctypes.POINTER(gespmm_plan_t)]
        L.gespmm_csr_simple.restype = ci
        L.gespmm_csr_simple.argtypes = [i64, i64, i64, vp, vp, vp, vp, vp, ci, vp]
        L.gespmm_csr_arg.restype = ci
        L.gespmm_csr_arg.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, vp, vp, ci, vp]
        L.gespmm_csr_transposed.restype = ci
        L.gespmm_csr_transposed.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, vp, ci, vp]
        L.gespmm_pool_backward.restype = ci
        L.gespmm_pool_backward.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, vp, vp]
        L.gespmm_csr_transpose_workspace_bytes.restype = ctypes.c_size_t
        L.gespmm_csr_transpose_workspace_bytes.argtypes = [i64]
        L.gespmm_csr_transpose.restype = ci
        L.gespmm_csr_transpose.argtypes = [i64, i64, i64, vp, vp, vp, ci, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.gespmm_csr_transpose_noalloc.restype = ci
        L.gespmm_csr_transpose_noalloc.argtypes = [i64, i64, i64, vp, vp, vp, ci, vp, vp, vp, vp]
        L.gespmm_csr_transpose_sorted_workspace_bytes.restype = ctypes.c_size_t
        L.gespmm_csr_transpose_sorted_workspace_bytes.argtypes = [i64, i64]
        L.gespmm_csr_transpose_sorted.restype = ci
        L.gespmm_csr_transpose_sorted.argtypes = [i64, i64, i64, vp, vp, vp, ci, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.gespmm_plan.restype = ci
        L.gespmm_plan.argtypes = [i64, i64, i64, ci, ctypes.POINTER(gespmm_plan_t)]
        tp = ctypes.POINTER(gespmm_tuning_t)
        L.gespmm_plan_ex.restype = ci
        L.gespmm_plan_ex.argtypes = [i64, i64, i64, i64, ci, ci, ctypes.c_size_t, tp, ctypes.POINTER(gespmm_plan_t)]
        L.gespmm_csr_workspace_bytes.restype = ctypes.c_size_t
        L.gespmm_csr_workspace_bytes.argtypes = [i64, i64, i64, i64, ci, tp]
        L.gespmm_csr_ex.restype = ci
        L.gespmm_csr_ex.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, ci, vp, ci, vp, ctypes.c_size_t, tp, vp, vp]
        L.gespmm_csr_arg_ex.restype = ci
        L.gespmm_csr_arg_ex.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, ci, vp, vp, ci, tp, vp]
        L.gespmm_csr_arg_ws.restype = ci
        L.gespmm_csr_arg_ws.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, ci, vp, vp, ci, vp, ctypes.c_size_t, tp, vp]
        L.gespmm_profiler_create.restype = ci
        L.gespmm_profiler_create.argtypes = [ci, ctypes.POINTER(vp)]
        L.gespmm_profiler_finish.restype = ci
        L.gespmm_profiler_finish.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int)]
        L.gespmm_calibration_copy.restype = ci
        L.gespmm_calibration_copy.argtypes = [vp, vp, i64, vp]
        L.gespmm_calibration_gather.restype = ci
        L.gespmm_calibration_gather.argtypes = [vp, i64, vp, i64, vp, i64, vp]
        L.gespmm_calibration_gather_shape.restype = ci
        L.gespmm_calibration_gather_shape.argtypes = [vp, i64, ci, vp, i64, ci, ci, ci, ci, vp, i64, vp]
        L.gespmm_custom_op_create.restype = ci
        L.gespmm_custom_op_create.argtypes = [ctypes.c_char_p, ctypes.c_char_p, ctypes.POINTER(vp), ctypes.c_char_p, ctypes.c_size_t]
        L.gespmm_custom_op_check.restype = ci
        L.gespmm_custom_op_check.argtypes = [ctypes.c_char_p, ctypes.c_char_p, ctypes.c_char_p, ctypes.c_char_p, ctypes.c_size_t]
        L.gespmm_custom_op_destroy.restype = ci
        L.gespmm_custom_op_destroy.argtypes = [vp]
        L.gespmm_csr_custom.restype = ci
        L.gespmm_csr_custom.argtypes = [vp, i64, i64, i64, i64, vp, vp, vp, vp, vp, tp, vp]
        L.gespmm_status_string.restype = ctypes.c_char_p
        L.gespmm_status_string.argtypes = [ci]
        L.gespmm_version.restype = ci
        _lib = L
    return _lib


def gespmm_status_string(status: int) -> str:
    return lib().gespmm_status_string(int(status)).decode()


def gespmm_version() -> int:
    return int(lib().gespmm_version())


def _check(status):
    if status != GESPMM_OK:
        raise GespmmError(status, gespmm_status_string(status))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check_tensors(rowptr, colind, vals, B, C, b_dtype=None):
    import torch
    b_dtype = b_dtype or torch.float32
    assert rowptr.is_cuda and rowptr.dtype == torch.int32 and rowptr.is_contiguous()
    assert colind.is_cuda and colind.dtype == torch.int32 and colind.is_contiguous()
    assert vals is None or (vals.is_cuda and vals.dtype == torch.float32 and vals.is_contiguous()
                            and vals.numel() == colind.numel())
    assert B.is_cuda and B.dtype == b_dtype and B.is_contiguous() and B.dim() == 2
    assert C.is_cuda and C.dtype == torch.float32 and C.is_contiguous() and C.dim() == 2
    assert C.shape == (rowptr.numel() - 1, B.shape[1])


def gespmm_csr(rowptr, colind, vals, B, op, C=None, stream=None):
    """C = A (x) B on the GPU; returns C (allocated here when not given)."""
    import torch
    M, (K, N) = rowptr.numel() - 1, B.shape
    if C is None:
        C = torch.empty((M, N), dtype=torch.float32, device=B.device)
    _check_tensors(rowptr, colind, vals, B, C)
    code = OPS[op] if isinstance(op, str) else int(op)
    _check(lib().gespmm_csr(M, K, N, colind.numel(), _ptr(rowptr), _ptr(colind), _ptr(vals),
                            _ptr(B), _ptr(C), code, _stream(stream)))
    return C


DTYPES = {"f32": 0, "bf16": 1, "f16": 2}


def gespmm_csr_b16(rowptr, colind, vals, B, op, C=None, stream=None):
    """C = A (x) B with B stored as torch.bfloat16 or torch.float16 (fp32 arithmetic and result)."""
    import torch
    M, (K, N) = rowptr.numel() - 1, B.shape
    if C is None:
        C = torch.empty((M, N), dtype=torch.float32, device=B.device)
    code_b = {torch.float32: 0, torch.bfloat16: 1, torch.float16: 2}[B.dtype]
    _check_tensors(rowptr, colind, vals, B, C, b_dtype=B.dtype)
    code = OPS[op] if isinstance(op, str) else int(op)
    _check(lib().gespmm_csr_b16(M, K, N, colind.numel(), _ptr(rowptr), _ptr(colind), _ptr(vals),
                                _ptr(B), code_b, _ptr(C), code, _stream(stream)))
    return C


def gespmm_csr_arg_b16(rowptr, colind, vals, B, op, C=None, arg=None, stream=None):
    """gespmm_csr_arg with B stored as torch.bfloat16 or torch.float16; returns (C fp32, arg int32)."""
    import torch
    M, (K, N) = rowptr.numel() - 1, B.shape
    if C is None:
        C = torch.empty((M, N), dtype=torch.float32, device=B.device)
    if arg is None:
        arg = torch.empty((M, N), dtype=torch.int32, device=B.device)
    code_b = {torch.float32: 0, torch.bfloat16: 1, torch.float16: 2}[B.dtype]
    _check_tensors(rowptr, colind, vals, B, C, b_dtype=B.dtype)
    assert arg.is_cuda and arg.dtype == torch.int32 and arg.is_contiguous() and arg.shape == C.shape
    code = OPS[op] if isinstance(op, str) else int(op)
    _check(lib().gespmm_csr_arg_b16(M, K, N, colind.numel(), _ptr(rowptr), _ptr(colind), _ptr(vals),
                                    _ptr(B), code_b, _ptr(C), _ptr(arg), code, _stream(stream)))
    return C, arg


def gespmm_plan_b16(M, N, nnz, b_dtype="bf16", aligned16=True) -> dict:
    p = gespmm_plan_t()
    _check(lib().gespmm_plan_b16(M, N, nnz, int(bool(aligned16)), DTYPES[b_dtype], ctypes.byref(p)))
    return {name: int(getattr(p, name)) for name, _ in p._fields_}


def gespmm_csr_simple(rowptr, colind, vals, B, op, C=None, stream=None):
    """Same as gespmm_csr, but the library reads nnz from rowptr[M] (one stream sync)."""
    import torch
    M, (K, N) = rowptr.numel() - 1, B.shape
    if C is None:
        C = torch.empty((M, N), dtype=torch.float32, device=B.device)
    _check_tensors(rowptr, colind, vals, B, C)
    code = OPS[op] if isinstance(op, str) else int(op)
    _check(lib().gespmm_csr_simple(M, K, N, _ptr(rowptr), _ptr(colind), _ptr(vals), _ptr(B),
                                   _ptr(C), code, _stream(stream)))
    return C


def gespmm_csr_arg(rowptr, colind, vals, B, op, C=None, arg=None, stream=None):
    """max / min and the position of the extreme; returns (C, arg) with arg int32 (M, N)."""
    import torch
    M, (K, N) = rowptr.numel() - 1, B.shape
    if C is None:
        C = torch.empty((M, N), dtype=torch.float32, device=B.device)
    if arg is None:
        arg = torch.empty((M, N), dtype=torch.int32, device=B.device)
    _check_tensors(rowptr, colind, vals, B, C)
    assert arg.is_cuda and arg.dtype == torch.int32 and arg.is_contiguous() and arg.shape == C.shape
    code = OPS[op] if isinstance(op, str) else int(op)
    _check(lib().gespmm_csr_arg(M, K, N, colind.numel(), _ptr(rowptr), _ptr(colind), _ptr(vals),
                                _ptr(B), _ptr(C), _ptr(arg), code, _stream(stream)))
    return C, arg


def gespmm_csr_transposed(rowptr, colind, vals, dC, op, K, dB=None, stream=None):
    """Gradient of sum / mean w.r.t. B from the CSR of A: dB = A^T (x) dC, shape (K, N)."""
    import torch
    M, N = dC.shape
    assert rowptr.numel() - 1 == M
    if dB is None:
        dB = torch.empty((K, N), dtype=torch.float32, device=dC.device)
    _check_tensors(rowptr, colind, vals, dC, dC)          # CSR arrays and dC as (M, N)
    assert dB.is_cuda and dB.dtype == torch.float32 and dB.is_contiguous() and dB.shape == (K, N)
    code = OPS[op] if isinstance(op, str) else int(op)
    _check(lib().gespmm_csr_transposed(M, K, N, colind.numel(), _ptr(rowptr), _ptr(colind), _ptr(vals),
                                       _ptr(dC), _ptr(dB), code, _stream(stream)))
    return dB


def gespmm_csr_transpose_workspace_bytes(K: int) -> int:
    return int(lib().gespmm_csr_transpose_workspace_bytes(int(K)))


def gespmm_csr_transpose(rowptr, colind, vals, K, scale_by_row_length=False, stream=None):
    """CSR arrays of the transposed matrix: returns (rowptrT, colindT, valsT) as new CUDA tensors
    (the workspace is a torch tensor allocated here; the library itself allocates nothing)."""
    import torch
    M, nnz = rowptr.numel() - 1, colind.numel()
    assert rowptr.is_cuda and rowptr.dtype == torch.int32 and rowptr.is_contiguous()
    assert colind.is_cuda and colind.dtype == torch.int32 and colind.is_contiguous()
    assert vals is None or (vals.is_cuda and vals.dtype == torch.float32 and vals.numel() == nnz)
    dev = rowptr.device
    rowptrT = torch.empty(K + 1, dtype=torch.int32, device=dev)
    colindT = torch.empty(nnz, dtype=torch.int32, device=dev)
    valsT = torch.empty(nnz, dtype=torch.float32, device=dev)
    nbytes = gespmm_csr_transpose_workspace_bytes(K)
    work = torch.empty(max(nbytes // 4, 1), dtype=torch.int32, device=dev)
    _check(lib().gespmm_csr_transpose(M, K, nnz, _ptr(rowptr), _ptr(colind), _ptr(vals),
                                      int(bool(scale_by_row_length)), _ptr(rowptrT), _ptr(colindT),
                                      _ptr(valsT), _ptr(work), nbytes, _stream(stream)))
    return rowptrT, colindT, valsT


def gespmm_csr_transpose_noalloc(rowptr, colind, vals, K, rowptrT, colindT, valsT, scale_by_row_length=False, stream=None):
    """gespmm_csr_transpose on the library's built-in scratch buffer: the caller passes inputs and the three
    output arrays (int32[K+1], int32[nnz], float32[nnz]); nothing is allocated, here or in the library."""
    import torch
    M, nnz = rowptr.numel() - 1, colind.numel()
    assert rowptr.is_cuda and rowptr.dtype == torch.int32 and rowptr.is_contiguous()
    assert colind.is_cuda and colind.dtype == torch.int32 and colind.is_contiguous()
    assert vals is None or (vals.is_cuda and vals.dtype == torch.float32 and vals.numel() == nnz)
    assert rowptrT.is_cuda and rowptrT.dtype == torch.int32 and rowptrT.is_contiguous() and rowptrT.numel() == K + 1
    assert colindT.is_cuda and colindT.dtype == torch.int32 and colindT.is_contiguous() and colindT.numel() == nnz
    assert valsT.is_cuda and valsT.dtype == torch.float32 and valsT.is_contiguous() and valsT.numel() == nnz
    _check(lib().gespmm_csr_transpose_noalloc(M, K, nnz, _ptr(rowptr), _ptr(colind), _ptr(vals),
                                              int(bool(scale_by_row_length)), _ptr(rowptrT), _ptr(colindT),
                                              _ptr(valsT), _stream(stream)))
    return rowptrT, colindT, valsT


def gespmm_csr_transpose_sorted_workspace_bytes(K: int, nnz: int) -> int:
    return int(lib().gespmm_csr_transpose_sorted_workspace_bytes(int(K), int(nnz)))


def gespmm_csr_transpose_sorted(rowptr, colind, vals, K, scale_by_row_length=False, stream=None):
    """CSR arrays of the transposed matrix by a stable radix sort on the columns (rows of A in
    increasing order inside every transposed row): returns (rowptrT, colindT, valsT).  The
    workspace (about 24 bytes per stored entry) is a torch tensor allocated here and released
    on return; the library itself allocates nothing."""
    import torch
    M, nnz = rowptr.numel() - 1, colind.numel()
    assert rowptr.is_cuda and rowptr.dtype == torch.int32 and rowptr.is_contiguous()
    assert colind.is_cuda and colind.dtype == torch.int32 and colind.is_contiguous()
    assert vals is None or (vals.is_cuda and vals.dtype == torch.float32 and vals.numel() == nnz)
    dev = rowptr.device
    rowptrT = torch.empty(K + 1, dtype=torch.int32, device=dev)
    colindT = torch.empty(nnz, dtype=torch.int32, device=dev)
    valsT = torch.empty(nnz, dtype=torch.float32, device=dev)
    nbytes = gespmm_csr_transpose_sorted_workspace_bytes(K, nnz)
    work = torch.empty(max(nbytes // 4, 1), dtype=torch.int32, device=dev)
    _check(lib().gespmm_csr_transpose_sorted(M, K, nnz, _ptr(rowptr), _ptr(colind), _ptr(vals),
                                             int(bool(scale_by_row_length)), _ptr(rowptrT), _ptr(colindT),
                                             _ptr(valsT), _ptr(work), nbytes, _stream(stream)))
    return rowptrT, colindT, valsT


def gespmm_pool_backward(colind, vals, arg, dC, K, dB=None, stream=None):
    """Gradient of max / min w.r.t. B routed through the positions `arg`; shape (K, N)."""
    import torch
    M, N = dC.shape
    if dB is None:
        dB = torch.empty((K, N), dtype=torch.float32, device=dC.device)
    assert arg.is_cuda and arg.dtype == torch.int32 and arg.is_contiguous() and arg.shape == dC.shape
    assert dC.is_cuda and dC.dtype == torch.float32 and dC.is_contiguous()
    assert dB.is_cuda and dB.dtype == torch.float32 and dB.is_contiguous() and dB.shape == (K, N)
    assert colind.is_cuda and colind.dtype == torch.int32 and colind.is_contiguous()
    assert vals is None or (vals.is_cuda and vals.dtype == torch.float32 and vals.numel() == colind.numel())
    _check(lib().gespmm_pool_backward(M, K, N, colind.numel(), _ptr(colind), _ptr(vals), _ptr(arg),
                                      _ptr(dC), _ptr(dB), _stream(stream)))
    return dB


def gespmm_plan(M, N, nnz, aligned16=True) -> dict:
    p = gespmm_plan_t()
    _check(lib().gespmm_plan(M, N, nnz, int(bool(aligned16)), ctypes.byref(p)))
    return {name: int(getattr(p, name)) for name, _ in p._fields_}


def gespmm_calibration_gather_shape(table, row_bytes, idx, lanes_per_row=8, load_bytes=16, in_flight=8, cache_policy=0,
                                    out=None, stream=None):
    """idx.numel() gathers of rows of `table` (a contiguous CUDA tensor cut into rows of row_bytes) with the
    given access shape; returns the scratch output tensor."""
    import torch
    nbytes = table.numel() * table.element_size()
    assert table.is_cuda and table.is_contiguous() and idx.is_cuda and idx.dtype == torch.int32 and idx.is_contiguous()
    if out is None:
        out = torch.empty(2048 * 256, dtype=torch.float32, device=table.device)
    _check(lib().gespmm_calibration_gather_shape(_ptr(table), nbytes, int(row_bytes), _ptr(idx), idx.numel(),
                                                 int(lanes_per_row), int(load_bytes), int(in_flight), int(cache_policy),
                                                 _ptr(out), out.numel() * out.element_size(), _stream(stream)))
    return out


def gespmm_plan_ex(M, K, N, nnz, b_dtype="f32", aligned16=True, workspace_bytes=0, tuning=None) -> dict:
    """The launch shape gespmm_csr_ex would use (workspace_bytes: what the caller will pass)."""
    p = gespmm_plan_t()
    _check(lib().gespmm_plan_ex(M, K, N, nnz, int(bool(aligned16)), DTYPES[b_dtype], int(workspace_bytes),
                                _tuning_ref(tuning), ctypes.byref(p)))
    return {name: int(getattr(p, name)) for name, _ in p._fields_}


def gespmm_csr_workspace_bytes(M, K, N, nnz, b_dtype="f32", tuning=None) -> int:
    return int(lib().gespmm_csr_workspace_bytes(M, K, N, nnz, DTYPES[b_dtype], _tuning_ref(tuning)))


def gespmm_csr_ex(rowptr, colind, vals, B, op, C=None, workspace=None, tuning=None, profiler=None, stream=None):
    """The forward call with its optional arguments: B float32 / bfloat16 / float16, `workspace` a CUDA tensor
    (enables the K-phased path), `tuning` overrides, `profiler` a handle from gespmm_profiler_create."""
    import torch
    M, (K, N) = rowptr.numel() - 1, B.shape
    if C is None:
        C = torch.empty((M, N), dtype=torch.float32, device=B.device)
    code_b = {torch.float32: 0, torch.bfloat16: 1, torch.float16: 2}[B.dtype]
    _check_tensors(rowptr, colind, vals, B, C, b_dtype=B.dtype)
    assert workspace is None or (workspace.is_cuda and workspace.is_contiguous())
    code = OPS[op] if isinstance(op, str) else int(op)
    _check(lib().gespmm_csr_ex(M, K, N, colind.numel(), _ptr(rowptr), _ptr(colind), _ptr(vals), _ptr(B), code_b,
                               _ptr(C), code, _ptr(workspace),
                               0 if workspace is None else workspace.numel() * workspace.element_size(),
                               _tuning_ref(tuning), profiler, _stream(stream)))
    return C


class gespmm_csr_prepared:
    """gespmm_csr_ex with its arguments checked and marshalled once, for loops that repeat one call (same tensors,
    same stream): calling the object issues the C call and returns C.  The tensors must stay alive and in place."""

    def __init__(self, rowptr, colind, vals, B, op, C=None, workspace=None, tuning=None, stream=None):
        import torch
        M, (K, N) = rowptr.numel() - 1, B.shape
        if C is None:
            C = torch.empty((M, N), dtype=torch.float32, device=B.device)
        code_b = {torch.float32: 0, torch.bfloat16: 1, torch.float16: 2}[B.dtype]
        _check_tensors(rowptr, colind, vals, B, C, b_dtype=B.dtype)
        assert workspace is None or (workspace.is_cuda and workspace.is_contiguous())
        code = OPS[op] if isinstance(op, str) else int(op)
        self.C = C
        self._keep = (rowptr, colind, vals, B, C, workspace, _tuning(tuning))
        self._fn = lib().gespmm_csr_ex
        self._head = (M, K, N, colind.numel(), _ptr(rowptr), _ptr(colind), _ptr(vals), _ptr(B), code_b, _ptr(C), code,
                      _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
                      None if self._keep[6] is None else ctypes.byref(self._keep[6]))
        self._stream = _stream(stream)

    def __call__(self, profiler=None):
        status = self._fn(*self._head, profiler, self._stream)
        if status != GESPMM_OK:
            _check(status)
        return self.C


def gespmm_csr_arg_ex(rowptr, colind, vals, B, op, C=None, arg=None, tuning=None, stream=None, workspace=None):
    """gespmm_csr_arg / gespmm_csr_arg_b16 with tuning overrides; returns (C fp32, arg int32).  With `workspace`
    (a device tensor of gespmm_csr_workspace_bytes(...) bytes) the call is gespmm_csr_arg_ws, which may take the
    K-phased path."""
    import torch
    M, (K, N) = rowptr.numel() - 1, B.shape
    if C is None:
        C = torch.empty((M, N), dtype=torch.float32, device=B.device)
    if arg is None:
        arg = torch.empty((M, N), dtype=torch.int32, device=B.device)
    code_b = {torch.float32: 0, torch.bfloat16: 1, torch.float16: 2}[B.dtype]
    _check_tensors(rowptr, colind, vals, B, C, b_dtype=B.dtype)
    assert arg.is_cuda and arg.dtype == torch.int32 and arg.is_contiguous() and arg.shape == C.shape
    code = OPS[op] if isinstance(op, str) else int(op)
    if workspace is not None:
        assert workspace.is_cuda and workspace.is_contiguous()
        _check(lib().gespmm_csr_arg_ws(M, K, N, colind.numel(), _ptr(rowptr), _ptr(colind), _ptr(vals), _ptr(B), code_b,
                                       _ptr(C), _ptr(arg), code, _ptr(workspace), workspace.numel() * workspace.element_size(),
                                       _tuning_ref(tuning), _stream(stream)))
        return C, arg
    _check(lib().gespmm_csr_arg_ex(M, K, N, colind.numel(), _ptr(rowptr), _ptr(colind), _ptr(vals), _ptr(B), code_b,
                                   _ptr(C), _ptr(arg), code, _tuning_ref(tuning), _stream(stream)))
    return C, arg


def gespmm_custom_op_create(source: str, name: str):
    """A user-defined reduce operation compiled at run time from HIP C++ text that defines the struct `name`
    (identity / step / merge).  Returns a handle for gespmm_csr_custom; a GespmmError carries the compiler's log."""
    handle = ctypes.c_void_p()
    log = ctypes.create_string_buffer(1 << 16)
    status = lib().gespmm_custom_op_create(source.encode(), name.encode(), ctypes.byref(handle), log, len(log))
    if status != GESPMM_OK:
        err = GespmmError(status, gespmm_status_string(status) + "\n" + log.value.decode(errors="replace"))
        err.log = log.value.decode(errors="replace")
        raise err
    return handle


def gespmm_custom_op_check(source: str, name: str, arch: str = "gfx950") -> str:
    """Compile the text of a user-defined reduce without a GPU; returns the compiler's messages (warnings) or
    raises GespmmError with them."""
    log = ctypes.create_string_buffer(1 << 16)
    status = lib().gespmm_custom_op_check(source.encode(), name.encode(), arch.encode(), log, len(log))
    if status != GESPMM_OK:
        err = GespmmError(status, gespmm_status_string(status) + "\n" + log.value.decode(errors="replace"))
        err.log = log.value.decode(errors="replace")
        raise err
    return log.value.decode(errors="replace")


def gespmm_custom_op_destroy(op):
    _check(lib().gespmm_custom_op_destroy(op))


def gespmm_csr_custom(op, rowptr, colind, vals, B, C=None, tuning=None, stream=None):
    """C = A (x) B with the reduce operation `op` (from gespmm_custom_op_create); fp32 tensors on the GPU."""
    import torch
    M, (K, N) = rowptr.numel() - 1, B.shape
    if C is None:
        C = torch.empty((M, N), dtype=torch.float32, device=B.device)
    _check_tensors(rowptr, colind, vals, B, C)
    _check(lib().gespmm_csr_custom(op, M, K, N, colind.numel(), _ptr(rowptr), _ptr(colind), _ptr(vals), _ptr(B), _ptr(C),
                                   _tuning_ref(tuning), _stream(stream)))
    return C


def gespmm_profiler_create(capacity: int):
    """A handle that owns `capacity` event pairs; pass it to gespmm_csr_ex, then to gespmm_profiler_finish."""
    handle = ctypes.c_void_p()
    _check(lib().gespmm_profiler_create(int(capacity), ctypes.byref(handle)))
    return handle


def gespmm_profiler_finish(handle):
    """Returns (summed main-kernel milliseconds, number of bracketed launches) and destroys the handle."""
    ms, n = ctypes.c_double(0.0), ctypes.c_int(0)
    _check(lib().gespmm_profiler_finish(handle, ctypes.byref(ms), ctypes.byref(n)))
    return float(ms.value), int(n.value)


def gespmm_calibration_copy(src, dst, stream=None):
    """dst <- src with the library's plain copy kernel (same-size contiguous CUDA tensors)."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes and src.is_contiguous() and dst.is_contiguous()
    _check(lib().gespmm_calibration_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream)))
    return dst


def gespmm_calibration_gather(table, idx, out=None, stream=None):
    """n = idx.numel() gathers of 128-byte lines of `table` (any contiguous CUDA tensor whose size is a
    multiple of 128 bytes); returns the scratch output tensor."""
    import torch
    nbytes = table.numel() * table.element_size()
    assert table.is_cuda and table.is_contiguous() and nbytes % 128 == 0
    assert idx.is_cuda and idx.dtype == torch.int32 and idx.is_contiguous()
    n = idx.numel()
    need = min((n + 255) // 256, 8192) * 4096
    if out is None:
        out = torch.empty(max(need // 4, 4), dtype=torch.float32, device=table.device)
    _check(lib().gespmm_calibration_gather(_ptr(table), nbytes // 128, _ptr(idx), n, _ptr(out),
                                           out.numel() * out.element_size(), _stream(stream)))
    return out
