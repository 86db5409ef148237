"""Pins for the CPU oracle: facts fixed by the paper's definition and by mathematics.

Each pin takes a callable  spmm(rowptr, colind, vals, B, op, rows=None) -> (Cref, Sabs)
and raises AssertionError when that callable is wrong.  The same list is run against
the real oracle (must pass) and against copies of it with one planted mistake each
(every copy must be rejected by at least one pin).

Nothing here retypes the oracle's loop: the expected values come from dense numpy
products, explicit per-entry Python folds, closed forms, scipy, or a hand-worked file.
"""
import math
import os

import numpy as np
import scipy.sparse as sp

import graphgen

OPS = ("sum", "mean", "max", "min")
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _py_fold(op, terms):
    """Fold Python floats (exact doubles) the way the definition says."""
    if not terms:
        return 0.0
    if op == "sum":
        return math.fsum(terms)
    if op == "mean":
        return math.fsum(terms) / len(terms)
    best = terms[0]
    for x in terms[1:]:
        if op == "max":
            if x > best or (x == best and math.copysign(1.0, x) > 0):
                best = x
        else:
            if x < best or (x == best and math.copysign(1.0, x) < 0):
                best = x
    return best


def _brute(rowptr, colind, vals, B, op):
    M = len(rowptr) - 1
    N = B.shape[1]
    C = np.zeros((M, N))
    S = np.zeros((M, N))
    for i in range(M):
        for j in range(N):
            terms = [float(vals[p]) * float(B[colind[p], j]) if vals is not None else float(B[colind[p], j])
                     for p in range(rowptr[i], rowptr[i + 1])]
            C[i, j] = _py_fold(op, terms)
            s = math.fsum(abs(t) for t in terms)
            S[i, j] = s / len(terms) if (op == "mean" and terms) else s
    return C, S


def _close(got, want, scale=None, tol=1e-12):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    bound = tol * (np.abs(want) if scale is None else np.asarray(scale)) + 1e-300
    assert np.all(np.isfinite(got)), "non-finite reference value"
    assert np.all(np.abs(got - want) <= bound), float(np.abs(got - want).max())


def _same_bits(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape
    assert np.array_equal(a.view(np.uint64), b.view(np.uint64))


# ---------------------------------------------------------------- pins -----
def pin_brute_force_tiny(spmm):
    """Per-entry Python folds on tiny matrices: empties, duplicates, unsorted, M != K."""
    cases = [dict(M=7, K=5, N=3, mean_len=2.0, seed=11, empty_frac=0.3, duplicates=True, sort_cols=False),
             dict(M=23, K=31, N=9, mean_len=4.0, seed=12, empty_frac=0.1),
             dict(M=40, K=17, N=1, mean_len=6.0, seed=13, duplicates=True),
             dict(M=5, K=64, N=4, mean_len=20.0, seed=14, sort_cols=False)]
    for c in cases:
        rp, ci, v = graphgen.random_csr(c["M"], c["K"], c["mean_len"], c["seed"],
                                        empty_frac=c.get("empty_frac", 0.0),
                                        duplicates=c.get("duplicates", False),
                                        sort_cols=c.get("sort_cols", True))
        B = graphgen.random_dense(c["K"], c["N"], c["seed"])
        for op in OPS:
            for vv in (v, None):
                want_c, want_s = _brute(rp, ci, vv, B, op)
                got_c, got_s = spmm(rp, ci, vv, B, op)
                if op in ("max", "min"):
                    _same_bits(got_c, want_c)
                else:
                    _close(got_c, want_c, scale=want_s + 1e-30)
                _close(got_s, want_s)


def pin_dense_matmul(spmm):
    """sum equals the float64 dense product A_dense @ B (duplicates added up in A_dense)."""
    rp, ci, v = graphgen.random_csr(33, 29, 5.0, 21, empty_frac=0.15, duplicates=True)
    B = graphgen.random_dense(29, 7, 21)
    A = np.zeros((33, 29))
    Aabs = np.zeros((33, 29))
    rows = np.repeat(np.arange(33), np.diff(rp))
    np.add.at(A, (rows, ci), v.astype(np.float64))
    np.add.at(Aabs, (rows, ci), np.abs(v.astype(np.float64)))
    want = A @ B.astype(np.float64)
    want_s = Aabs @ np.abs(B.astype(np.float64))
    got_c, got_s = spmm(rp, ci, v, B, "sum")
    _close(got_c, want, scale=want_s + 1e-30)
    _close(got_s, want_s)
    lens = np.diff(rp).astype(np.float64)[:, None]
    got_m, got_ms = spmm(rp, ci, v, B, "mean")
    safe = np.where(lens == 0, 1.0, lens)
    _close(got_m, want / safe, scale=want_s / safe + 1e-30)
    _close(got_ms, want_s / safe)


def pin_identity(spmm):
    """A = I gives C == B bit-for-bit for every op."""
    M, N = 19, 6
    rp = np.arange(M + 1, dtype=np.int32)
    ci = np.arange(M, dtype=np.int32)
    B = graphgen.random_dense(M, N, 31)
    for op in OPS:
        for v in (np.ones(M, dtype=np.float32), None):
            got_c, got_s = spmm(rp, ci, v, B, op)
            _same_bits(got_c, B.astype(np.float64))
            _same_bits(got_s, np.abs(B.astype(np.float64)))


def pin_all_ones_B(spmm):
    """All-ones B: sum = weighted row sum, mean = that / len, max/min = extreme stored value."""
    rp, ci, v = graphgen.random_csr(50, 40, 5.0, 41, empty_frac=0.2, duplicates=True, sort_cols=False)
    B = np.ones((40, 5), dtype=np.float32)
    for vv in (v, None):
        for op in OPS:
            got_c, _ = spmm(rp, ci, vv, B, op)
            for i in range(50):
                row = ([float(x) for x in vv[rp[i]:rp[i + 1]]] if vv is not None
                       else [1.0] * int(rp[i + 1] - rp[i]))
                want = _py_fold(op, row)
                _close(got_c[i], np.full(5, want), scale=np.full(5, math.fsum(map(abs, row)) + 1e-30))
    # unweighted: sum == degree, mean == 1 for non-empty rows
    got_c, _ = spmm(rp, ci, None, B, "sum")
    _same_bits(got_c[:, 0], np.diff(rp).astype(np.float64))
    got_m, _ = spmm(rp, ci, None, B, "mean")
    _same_bits(got_m[:, 0], (np.diff(rp) > 0).astype(np.float64))


def pin_closed_form_long_row(spmm):
    """One dense row of n ones against B[k, j] = k * (j + 1): arithmetic-series closed forms."""
    n, N = 100_000, 3
    rp = np.array([0, n, n], dtype=np.int32)          # second row empty
    ci = np.arange(n, dtype=np.int32)
    B = (np.arange(n, dtype=np.float64)[:, None] * (np.arange(N) + 1.0)[None, :]).astype(np.float32)
    tri = n * (n - 1) // 2
    for v in (np.ones(n, dtype=np.float32), None):
        c, s = spmm(rp, ci, v, B, "sum")
        _same_bits(c[0], np.array([tri * (j + 1) for j in range(N)], dtype=np.float64))
        _same_bits(s[0], c[0])
        c, _ = spmm(rp, ci, v, B, "mean")
        _same_bits(c[0], np.array([(n - 1) / 2 * (j + 1) for j in range(N)]))
        c, _ = spmm(rp, ci, v, B, "max")
        _same_bits(c[0], np.array([(n - 1) * (j + 1) for j in range(N)], dtype=np.float64))
        c, _ = spmm(rp, ci, v, B, "min")
        _same_bits(c[0], np.zeros(N))
        _same_bits(c[1], np.zeros(N))


def pin_negative_rows_and_signed_zero(spmm):
    """max of an all-negative row stays negative; +0 beats -0 for max and loses for min."""
    rp = np.array([0, 3, 5, 7], dtype=np.int32)
    ci = np.array([0, 1, 2, 3, 4, 4, 3], dtype=np.int32)
    v = np.array([1, 2, 0.5, 1, 1, 1, 1], dtype=np.float32)
    B = np.array([[-3.0], [-1.0], [-8.0], [-0.0], [0.0]], dtype=np.float32)
    c, _ = spmm(rp, ci, v, B, "max")
    _same_bits(c[:, 0], np.array([-2.0, 0.0, 0.0]))
    c, _ = spmm(rp, ci, v, B, "min")
    _same_bits(c[:, 0], np.array([-4.0, -0.0, -0.0]))
    c, _ = spmm(rp, ci, v, -B, "min")
    _same_bits(c[0], np.array([2.0]))


def pin_hand_worked(spmm):
    """Values typed in by hand (tests/golden/hand_worked_4x5.txt)."""
    rec = {}
    with open(os.path.join(GOLDEN, "hand_worked_4x5.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                rec[line[0]] = [float(x) for x in line[1:]]
    rp = np.array(rec["rowptr"], dtype=np.int32)
    ci = np.array(rec["colind"], dtype=np.int32)
    v = np.array(rec["vals"], dtype=np.float32)
    B = np.array(rec["B"], dtype=np.float32).reshape(5, 2)
    for op in OPS:
        c, s = spmm(rp, ci, v, B, op)
        _close(c, np.array(rec[op]).reshape(4, 2), tol=1e-15)
        if op == "sum":
            _close(s, np.array(rec["sabs_sum"]).reshape(4, 2), tol=1e-15)


def pin_scipy_float64(spmm):
    """sum on power-law graphs equals scipy's CSR product carried out in float64."""
    for w in (graphgen.workload(0), graphgen.workload(1, 0.25), graphgen.workload(2, 0.02)):
        N = 8
        B = w.B(N)
        A = sp.csr_matrix((w.vals.astype(np.float64), w.colind, w.rowptr), shape=(w.M, w.K))
        Aabs = sp.csr_matrix((np.abs(w.vals.astype(np.float64)), w.colind, w.rowptr), shape=(w.M, w.K))
        want = A @ B.astype(np.float64)
        want_s = Aabs @ np.abs(B.astype(np.float64))
        c, s = spmm(w.rowptr, w.colind, w.vals, B, "sum")
        _close(c, want, scale=want_s + 1e-30)
        _close(s, want_s)


def pin_invariants(spmm):
    """Column independence, in-row permutation, max/min duality, mean * len == sum, row subsets."""
    M, K, N = 60, 45, 9
    rp, ci, v = graphgen.random_csr(M, K, 6.0, 51, empty_frac=0.1)
    B = graphgen.random_dense(K, N, 51)
    rng = np.random.default_rng(7)
    ci2, v2 = ci.copy(), v.copy()
    for i in range(M):
        perm = rng.permutation(rp[i + 1] - rp[i]) + rp[i]
        ci2[rp[i]:rp[i + 1]] = ci[perm]
        v2[rp[i]:rp[i + 1]] = v[perm]
    for op in OPS:
        full, fs = spmm(rp, ci, v, B, op)
        for j0, j1 in ((0, 4), (4, 9), (8, 9)):
            part, ps = spmm(rp, ci, v, np.ascontiguousarray(B[:, j0:j1]), op)
            _same_bits(part, full[:, j0:j1])
            _same_bits(ps, fs[:, j0:j1])
        shuffled, _ = spmm(rp, ci2, v2, B, op)
        if op in ("max", "min"):
            _same_bits(shuffled, full)
        else:
            _close(shuffled, full, scale=fs + 1e-30)
        rows = np.array([M - 1, 0, 17, 17, 3], dtype=np.int64)
        sub, ss = spmm(rp, ci, v, B, op, rows=rows)
        _same_bits(sub, full[rows])
        _same_bits(ss, fs[rows])
    mx, _ = spmm(rp, ci, v, B, "max")
    mn, _ = spmm(rp, ci, v, -B, "min")
    nonempty = np.diff(rp) > 0            # an empty row is +0 on both sides, so -(+0) would differ
    _same_bits(mx[nonempty], -mn[nonempty])
    sm, ss = spmm(rp, ci, v, B, "sum")
    me, _ = spmm(rp, ci, v, B, "mean")
    lens = np.diff(rp).astype(np.float64)[:, None]
    _close(me * lens, sm, scale=ss + 1e-30)
    # unweighted: min <= mean <= max element-wise on non-empty rows
    lo, _ = spmm(rp, ci, None, B, "min")
    hi, _ = spmm(rp, ci, None, B, "max")
    mid, _ = spmm(rp, ci, None, B, "mean")
    assert np.all(lo <= mid + 1e-15) and np.all(mid <= hi + 1e-15)


PINS = (pin_brute_force_tiny, pin_dense_matmul, pin_identity, pin_all_ones_B,
        pin_closed_form_long_row, pin_negative_rows_and_signed_zero, pin_hand_worked,
        pin_scipy_float64, pin_invariants)
