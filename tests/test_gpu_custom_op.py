"""User-defined reduce operations (include/gespmm_custom.hpp) on the GPU against the general fold
of the CPU oracle.  The two example operations live in tests/custom_ops/custom_ops.hip."""
import ctypes
import os

import numpy as np
import pytest

import graphgen
import oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

LIB = os.path.join(os.path.dirname(os.path.abspath(__file__)), "custom_ops", "libcustom_ops.so")


@pytest.fixture(scope="module")
def custom():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    if not os.path.exists(LIB):                      # normally built beforehand by __graft_entry__.build()
        from paper_2007_03179_amd import build as hip_build
        hip_build.build_custom_example(force=True)
    L = ctypes.CDLL(LIB)
    i64, vp = ctypes.c_int64, ctypes.c_void_p
    for name in ("custom_sum_of_squares", "custom_max_magnitude"):
        fn = getattr(L, name)
        fn.restype = ctypes.c_int
        fn.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, vp, vp]
    return L


def run(fn, rp, ci, v, B):
    d = lambda x: None if x is None else torch.from_numpy(np.ascontiguousarray(x)).cuda()
    d_rp, d_ci, d_v, d_B = d(rp), d(ci), d(v), d(B)
    C = torch.full((len(rp) - 1, B.shape[1]), float("nan"), dtype=torch.float32, device="cuda")
    p = lambda t: None if t is None else ctypes.c_void_p(t.data_ptr())
    st = fn(len(rp) - 1, B.shape[0], B.shape[1], len(ci), p(d_rp), p(d_ci), p(d_v), p(d_B), p(C),
            ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == 0, st
    torch.cuda.synchronize()
    return C.cpu().numpy()


@pytest.mark.parametrize("N", [3, 8, 64, 160])
def test_user_defined_reduce_matches_general_fold(custom, N):
    # short rows, empty rows, and one row spanning many chunks (combined by the CAS loop)
    rp, ci, v = graphgen.random_csr(400, 300, 6.0, 500 + N, empty_frac=0.1, long_rows=((33, 1500),), duplicates=True)
    B = graphgen.random_dense(300, N, N)
    for vv in (v, None):
        print(f"  case custom N={N} vals={'given' if vv is not None else 'NULL'}", flush=True)
        got = run(custom.custom_sum_of_squares, rp, ci, vv, B)
        ref = oracle.spmm_custom(rp, ci, vv, B, 0.0, lambda acc, a, b: acc + (a * b) ** 2)
        assert np.all(np.abs(got - ref) <= 1e-5 * ref + 1e-6), float(np.abs(got - ref).max())
        got = run(custom.custom_max_magnitude, rp, ci, vv, B)
        ref = oracle.spmm_custom(rp, ci, vv, B, 0.0, lambda acc, a, b: max(acc, abs(a * b)))
        assert np.array_equal(got.view(np.uint32), ref.astype(np.float32).view(np.uint32))


def test_user_defined_reduce_argument_errors(custom):
    p = ctypes.c_void_p(0x1000)
    assert custom.custom_sum_of_squares(-1, 4, 4, 0, p, p, p, p, p, None) == 1
    assert custom.custom_sum_of_squares(4, 4, 4, 8, None, p, p, p, p, None) == 2
    assert custom.custom_max_magnitude(0, 4, 4, 0, p, p, p, p, p, None) == 0
