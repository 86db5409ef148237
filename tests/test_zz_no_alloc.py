"""The entry point that allocates nothing (gespmm_csr_transpose_noalloc) against the entry point it is a
variant of (gespmm_csr_transpose, caller-provided workspace) and against the CPU oracle, through the C ABI.

Index work: compared exactly.  The order inside a transposed row is unspecified for both entry points, so
rows are compared as sorted lists of (row index of A, value bits); the row starts are compared as they are.
Two calls in a row share the library's built-in scratch buffer; the second has the smaller input.
"""
import ctypes
import sys

import numpy as np
import pytest

import graphgen
import oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gs():
    import paper_2007_03179_amd as gs
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    gs.lib()
    return gs


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def canonical(rowptrT, colindT, valsT):
    """Entries of every transposed row sorted by (row index of A, value bits)."""
    rowptrT = np.asarray(rowptrT)
    row_of = np.repeat(np.arange(len(rowptrT) - 1), np.diff(rowptrT))
    order = np.lexsort((np.asarray(valsT).view(np.uint32), np.asarray(colindT), row_of))
    return np.asarray(colindT)[order], np.asarray(valsT).view(np.uint32)[order]


def transpose_both_ways(gs, rp, ci, v, K, scale, label):
    say(f"  case no-alloc {label} M={len(rp) - 1} K={K} nnz={len(ci)} scale={scale} vals={'NULL' if v is None else 'given'}")
    d_rp, d_ci = torch.from_numpy(rp).cuda(), torch.from_numpy(ci).cuda()
    d_v = None if v is None else torch.from_numpy(v).cuda()
    outs = (torch.full((K + 1,), -7, dtype=torch.int32, device="cuda"),
            torch.full((len(ci),), -7, dtype=torch.int32, device="cuda"),
            torch.full((len(ci),), float("nan"), dtype=torch.float32, device="cuda"))
    torch.cuda.synchronize()
    gs.gespmm_csr_transpose_noalloc(d_rp, d_ci, d_v, K, *outs, scale_by_row_length=scale)
    torch.cuda.synchronize()
    got = [x.cpu().numpy() for x in outs]
    want = [x.cpu().numpy() for x in gs.gespmm_csr_transpose(d_rp, d_ci, d_v, K, scale_by_row_length=scale)]
    ref = oracle.csr_transpose(rp, ci, v, K, scale_by_row_length=scale)
    for other, name in ((want, "gespmm_csr_transpose"), (ref, "oracle")):
        assert np.array_equal(got[0], other[0]), f"{label}: row starts differ from {name}"
        a, b = canonical(*got), canonical(*other)
        assert np.array_equal(a[0], b[0]), f"{label}: row indices differ from {name}"
        assert np.array_equal(a[1], b[1]), f"{label}: value bits differ from {name}"


def test_two_calls_in_a_row_second_one_smaller(gs):
    big = graphgen.random_csr(6000, 5000, 14.0, 41, empty_frac=0.1, long_rows=((3, 7000), (4000, 2500)), duplicates=True)
    small = graphgen.random_csr(300, 170, 5.0, 42, empty_frac=0.3, long_rows=((9, 600),))
    transpose_both_ways(gs, *big, 5000, False, "first (larger)")
    transpose_both_ways(gs, *small, 170, True, "second (smaller)")
    transpose_both_ways(gs, big[0], big[1], None, 5000, True, "third (larger again, vals NULL)")


def test_workload_size_and_empty_input(gs):
    w = graphgen.workload(2)                                      # 169,343 columns, 2.33 M entries
    transpose_both_ways(gs, w.rowptr, w.colind, w.vals, w.K, True, w.name)
    rp = np.zeros(6, dtype=np.int32)                              # no entries at all: every row start is 0
    transpose_both_ways(gs, rp, np.zeros(0, np.int32), np.zeros(0, np.float32), 9, False, "nnz=0")


def test_limit_is_enforced_on_the_host(gs):
    L = gs.lib()
    p = ctypes.c_void_p(0x1000)
    limit = 2097152                                               # GESPMM_NOALLOC_TRANSPOSE_MAX_K
    assert L.gespmm_csr_transpose_noalloc(4, limit + 1, 8, p, p, p, 0, p, p, p, None) == 6
    assert "scratch" in gs.gespmm_status_string(6)
    assert L.gespmm_csr_transpose_noalloc(4, 4, 8, p, p, p, 0, None, p, p, None) == 2
    assert L.gespmm_csr_transpose_noalloc(4, -1, 8, p, p, p, 0, p, p, p, None) == 1
