"""Seeded input generator: determinism, structure and the stated workload shapes (CPU only)."""
import numpy as np
import pytest

import graphgen


def _check_csr(M, K, rp, ci, symmetric=False, no_self_loops=False):
    assert rp.dtype == np.int32 and ci.dtype == np.int32
    assert rp.shape == (M + 1,) and rp[0] == 0 and rp[-1] == ci.shape[0]
    lens = np.diff(rp)
    assert (lens >= 0).all()
    assert ci.size == 0 or (ci.min() >= 0 and ci.max() < K)
    rows = np.repeat(np.arange(M, dtype=np.int64), lens)
    keys = rows * K + ci
    assert (np.diff(keys) > 0).all(), "columns must be sorted and unique inside every row"
    if no_self_loops:
        assert (rows != ci).all()
    if symmetric:
        assert np.array_equal(np.sort(ci.astype(np.int64) * K + rows), keys)


def test_tiny_and_sweep_have_exact_sizes():
    w0 = graphgen.workload(0)
    assert (w0.M, w0.K, w0.nnz) == (2708, 2708, 10556)
    _check_csr(w0.M, w0.K, w0.rowptr, w0.colind, symmetric=True, no_self_loops=True)
    d = np.diff(w0.rowptr).astype(np.float64)
    i, j = np.repeat(np.arange(w0.M), np.diff(w0.rowptr)), w0.colind
    np.testing.assert_allclose(w0.vals, 1.0 / np.sqrt(d[i] * d[j]), rtol=1e-6)
    w1 = graphgen.workload(1)
    assert (w1.M, w1.nnz) == (19717, 88648)
    _check_csr(w1.M, w1.K, w1.rowptr, w1.colind, symmetric=True, no_self_loops=True)
    assert w1.vals.min() > 0 and w1.vals.max() <= 1
    assert w1.widths == (32, 64, 128, 256, 512)


def test_general_ops_workload_shape():
    w = graphgen.workload(2)
    assert w.M == 169343 and abs(w.nnz - 2.33e6) < 0.02e6
    _check_csr(w.M, w.K, w.rowptr, w.colind, no_self_loops=True)
    lens = np.diff(w.rowptr)
    assert 0.03 <= (lens == 0).mean() < 0.04
    assert lens.max() > 20 * lens.mean()            # power-law skew
    assert (w.vals == 1).all()
    B = w.B(128)
    assert B.shape == (w.K, 128) and abs(B.mean()) < 0.01 and abs(B.std() - 1) < 0.01
    assert (B != 0).all()


def test_scaled_large_and_skew_workloads():
    w = graphgen.workload(3, 0.01)
    _check_csr(w.M, w.K, w.rowptr, w.colind, symmetric=True, no_self_loops=True)
    assert np.diff(w.rowptr).mean() > 100
    w = graphgen.workload(4, 0.01)
    _check_csr(w.M, w.K, w.rowptr, w.colind)
    lens = np.diff(w.rowptr)
    assert (lens == 0).mean() >= 0.05
    assert lens.max() > 50 * lens.mean()
    # hub rows sit at low ids (rows are not permuted)
    assert lens[: w.M // 16].sum() > lens[-(w.M // 16):].sum() * 10


def test_same_seed_same_graph_any_thread_count():
    a = graphgen.workload(2, 0.05)
    graphgen.set_threads(1)
    try:
        b = graphgen.workload(2, 0.05)
        r1 = graphgen.rmat(5000, 13, 40000, seed=9)
        u1 = graphgen.uniform_pm1((1000, 7), 5, stream=7)
    finally:
        graphgen.set_threads(8)
    assert np.array_equal(a.rowptr, b.rowptr) and np.array_equal(a.colind, b.colind)
    r8 = graphgen.rmat(5000, 13, 40000, seed=9)
    assert np.array_equal(r1[2], r8[2]) and np.array_equal(r1[3], r8[3])
    assert np.array_equal(u1, graphgen.uniform_pm1((1000, 7), 5, stream=7))
    other = graphgen.rmat(5000, 13, 40000, seed=10)
    assert not np.array_equal(r1[3][:1000], other[3][:1000])


def test_value_fillers():
    u = graphgen.uniform_pm1((4096, 16), 3)
    assert u.min() > -1 and u.max() < 1 and (u != 0).all() and abs(u.mean()) < 0.02
    p = graphgen.uniform_01(100000, 3)
    assert p.min() > 0 and p.max() <= 1 and abs(p.mean() - 0.5) < 0.01
    n = graphgen.normal((100000,), 3)
    assert abs(n.mean()) < 0.02 and abs(n.std() - 1) < 0.02


@pytest.mark.parametrize("kw", [dict(duplicates=True, sort_cols=False), dict(empty_frac=0.5),
                                dict(long_rows=((3, 500),))])
def test_random_csr_is_valid(kw):
    rp, ci, v = graphgen.random_csr(50, 700, 5.0, 1, **kw)
    assert rp[0] == 0 and rp[-1] == ci.shape[0] == v.shape[0]
    assert (np.diff(rp) >= 0).all() and ci.min() >= 0 and ci.max() < 700
    if "long_rows" in kw:
        assert rp[4] - rp[3] == 500


def test_uniform_random_extra_workload():
    w = graphgen.workload("uniform_random_65k")
    _check_csr(w.M, w.K, w.rowptr, w.colind)
    lens = np.diff(w.rowptr)
    assert w.M == 65536 and abs(w.nnz - 650_000) < 5_000
    assert lens.max() < 40 and abs(lens.mean() - 9.9) < 0.2       # no skew


def test_matrix_market_reader_against_scipy(tmp_path):
    import scipy.io
    import scipy.sparse as sp
    from graphgen.mtx import read_matrix_market
    rng = np.random.default_rng(0)
    A = sp.random(37, 23, density=0.15, random_state=1, format="coo")
    A.data = np.round(A.data * 100) / 4
    scipy.io.mmwrite(str(tmp_path / "general.mtx"), A)
    S = sp.random(19, 19, density=0.2, random_state=2, format="coo")
    S = sp.coo_matrix(sp.triu(S) + sp.triu(S, 1).T)
    scipy.io.mmwrite(str(tmp_path / "symmetric.mtx"), S, symmetry="symmetric")
    P = sp.coo_matrix((np.ones(5), ([0, 3, 3, 6, 6], [1, 0, 4, 2, 6])), shape=(7, 7))
    scipy.io.mmwrite(str(tmp_path / "pattern.mtx"), P, field="pattern")
    for name, ref in (("general", A), ("symmetric", S), ("pattern", P)):
        M, K, rp, ci, v = read_matrix_market(tmp_path / f"{name}.mtx")
        assert (M, K) == ref.shape and rp.dtype == np.int32 and ci.dtype == np.int32 and v.dtype == np.float32
        got = sp.csr_matrix((v.astype(np.float64), ci, rp), shape=(M, K))
        assert abs(got - sp.csr_matrix(scipy.io.mmread(str(tmp_path / f"{name}.mtx")))).max() < 1e-6
        rows = np.repeat(np.arange(M), np.diff(rp))
        assert (np.diff(rows * K + ci) > 0).all()
    (tmp_path / "bad.mtx").write_text("%%MatrixMarket matrix array real general\n2 2\n1\n2\n3\n4\n")
    with pytest.raises(ValueError):
        read_matrix_market(tmp_path / "bad.mtx")


def test_grid_stencils_have_the_textbook_structure():
    for n in (1, 2, 7):
        M, K, rp, ci = graphgen.grid2d(n)
        _check_csr(M, K, rp, ci)
        assert M == n * n and ci.shape[0] == 5 * n * n - 4 * n            # n^2 centres + 4 n (n - 1) neighbours
    for n in (1, 3, 5):
        M, K, rp, ci = graphgen.grid3d(n)
        _check_csr(M, K, rp, ci)
        assert M == n ** 3 and ci.shape[0] == (3 * n - 2) ** 3            # product of the 1-D counts 3 n - 2
    M, K, rp, ci = graphgen.grid2d(4)
    A = np.zeros((16, 16), dtype=int)
    A[np.repeat(np.arange(16), np.diff(rp)), ci] = 1
    assert (A == A.T).all() and A[5].nonzero()[0].tolist() == [1, 4, 5, 6, 9] and A[0].nonzero()[0].tolist() == [0, 1, 4]
    M, K, rp, ci = graphgen.grid3d(3)
    assert rp[14] - rp[13] == 27 and rp[1] - rp[0] == 8                   # centre cell, corner cell


def test_shape_suite_is_seeded_and_valid():
    for name in ("powerlaw_30k_d8", "rmat_64k_d16", "grid2d_300"):
        a, b = graphgen.suite_matrix(name), graphgen.suite_matrix(name)
        _check_csr(a.M, a.K, a.rowptr, a.colind)
        assert a.describe()["csr_hash"] == b.describe()["csr_hash"] and a.widths == (128, 256, 512)
        assert a.vals.min() > 0 and a.vals.max() <= 1
    assert len(graphgen.SUITE_NAMES) == 16
