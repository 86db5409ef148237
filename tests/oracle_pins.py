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
    """Column independence, in-row permutation, max/min duality, mean * len == sum, row subsets,
    min <= mean <= max, linearity in B, row-permutation equivariance."""
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
    # linearity in B for sum and mean (values chosen so that B1 + B2 is exact in fp32)
    B1 = np.round(B * 64).astype(np.float32) / 64
    B2 = np.round(graphgen.random_dense(K, N, 52) * 64).astype(np.float32) / 64
    for op in ("sum", "mean"):
        both, bs = spmm(rp, ci, v, B1 + B2, op)
        one, s1 = spmm(rp, ci, v, B1, op)
        two, s2 = spmm(rp, ci, v, B2, op)
        _close(both, one + two, scale=s1 + s2 + 1e-30)
    # permuting the rows of A permutes the rows of C (all ops, bit for bit)
    order = rng.permutation(M)
    lens_i = np.diff(rp)
    rp3 = np.zeros(M + 1, dtype=np.int32)
    np.cumsum(lens_i[order], out=rp3[1:])
    ci3 = np.concatenate([ci[rp[i]:rp[i + 1]] for i in order]).astype(np.int32)
    v3 = np.concatenate([v[rp[i]:rp[i + 1]] for i in order]).astype(np.float32)
    for op in OPS:
        moved, ms = spmm(rp3, ci3, v3, B, op)
        plain, ps = spmm(rp, ci, v, B, op)
        _same_bits(moved, plain[order])
        _same_bits(ms, ps[order])


PINS = (pin_brute_force_tiny, pin_dense_matmul, pin_identity, pin_all_ones_B,
        pin_closed_form_long_row, pin_negative_rows_and_signed_zero, pin_hand_worked,
        pin_scipy_float64, pin_invariants)


# ------------------------------------------------ gradient-side pins -------
# These take the oracle module (or an object with the same functions):
#   O.spmm, O.spmm_arg, O.spmm_transposed, O.pool_backward
def _brute_arg(rowptr, colind, vals, B, op):
    """Value: extreme of the exact products (Python floats), +0 above -0.  Position: the first stored entry
    whose product, rounded once to fp32 (numpy's fp32 multiply of the two fp32 factors), has the bits of
    the value rounded once to fp32."""
    M, N = len(rowptr) - 1, B.shape[1]
    C = np.zeros((M, N))
    arg = np.full((M, N), -1, dtype=np.int32)
    one = np.float32(1.0)
    for i in range(M):
        for j in range(N):
            ps = range(rowptr[i], rowptr[i + 1])
            if not len(ps):
                continue
            exact = [(float(vals[p]) if vals is not None else 1.0) * float(B[colind[p], j]) for p in ps]
            keys = [(x, math.copysign(1.0, x)) for x in exact]
            best = exact[keys.index(max(keys) if op == "max" else min(keys))]
            target = np.float32(best).view(np.uint32)
            rounded = [((vals[p] if vals is not None else one) * B[colind[p], j]).view(np.uint32) for p in ps]
            C[i, j], arg[i, j] = best, ps[rounded.index(target)]
    return C, arg


def pin_arg_ties_inside_one_fp32_rounding_interval(O):
    """Two stored entries whose exact products differ by 2^-46 and round to the same fp32 number: they are
    equals for the position (it refers to the fp32 result), so the one stored first wins, also when its
    exact product is the smaller (max) or the larger (min) of the two."""
    e = 2.0 ** -23
    rp = np.array([0, 3, 3, 6], dtype=np.int32)
    ci = np.array([0, 1, 2, 2, 1, 0], dtype=np.int32)
    # row 0 stores (1 + 2e) * 1 first, then (1 + e) * (1 + e) = 1 + 2e + e^2, then a smaller term;
    # row 2 stores them in the opposite order
    B = np.array([[1.0], [1.0 + e], [0.5]], dtype=np.float32)
    v = np.array([1.0 + 2 * e, 1.0 + e, 1.0, 1.0, 1.0 + e, 1.0 + 2 * e], dtype=np.float32)
    assert float(v[0]) * float(B[0, 0]) < float(v[1]) * float(B[1, 0])            # exact products differ ...
    assert v[0] * B[0, 0] == v[1] * B[1, 0]                                         # ... their fp32 roundings do not
    c, a = O.spmm_arg(rp, ci, v, B, "max")
    assert a[:, 0].tolist() == [0, -1, 4] and c[0, 0] == c[2, 0] == (1.0 + e) * (1.0 + e) and c[1, 0] == 0.0
    c, a = O.spmm_arg(rp, ci, -v, B, "min")
    assert a[:, 0].tolist() == [0, -1, 4] and c[0, 0] == -(1.0 + e) * (1.0 + e)
    want_c, want_a = _brute_arg(rp, ci, v, B, "max")
    assert np.array_equal(want_a, np.array([[0], [-1], [4]])) and want_c[0, 0] == (1.0 + e) * (1.0 + e)


def pin_arg_brute_force_with_ties(O):
    """Position of the extreme: per-entry Python scan; ties must go to the first stored entry."""
    rp, ci, v = graphgen.random_csr(30, 12, 5.0, 61, empty_frac=0.2, duplicates=True, sort_cols=False)
    B = np.round(graphgen.random_dense(12, 4, 61) * 3.0).astype(np.float32)      # few distinct values: ties
    v = np.round(v * 2.0).astype(np.float32)
    v[v == 0] = 1.0
    B[3] = 0.0
    B[4] = -0.0
    for op in ("max", "min"):
        for vv in (v, None):
            want_c, want_a = _brute_arg(rp, ci, vv, B, op)
            got_c, got_a = O.spmm_arg(rp, ci, vv, B, op)
            _same_bits(got_c, want_c)
            assert np.array_equal(got_a, want_a)
            ties = 0
            for i in range(30):
                for j in range(4):
                    prods = [(float(vv[p]) if vv is not None else 1.0) * float(B[ci[p], j]) for p in range(rp[i], rp[i + 1])]
                    ties += prods.count(want_c[i, j]) > 1
            assert ties > 5, "the case must contain ties to mean anything"
    rows = np.array([7, 0, 29], dtype=np.int64)
    full_c, full_a = O.spmm_arg(rp, ci, v, B, "max")
    sub_c, sub_a = O.spmm_arg(rp, ci, v, B, "max", rows=rows)
    _same_bits(sub_c, full_c[rows])
    assert np.array_equal(sub_a, full_a[rows])


def pin_arg_consistent_with_forward(O):
    """The value at the reported position is the forward result, and the position lies in the row."""
    w = graphgen.workload(2, 0.01)
    B = w.B(5)
    vals = graphgen.uniform_pm1(w.nnz, 77)
    for op in ("max", "min"):
        c_fwd, _ = O.spmm(w.rowptr, w.colind, vals, B, op)
        c, a = O.spmm_arg(w.rowptr, w.colind, vals, B, op)
        _same_bits(c, c_fwd)
        lens = np.diff(w.rowptr)
        assert np.all(a[lens == 0] == -1) and np.all(a[lens > 0] >= 0)
        i, j = np.nonzero(a >= 0)
        p = a[i, j]
        assert np.all(p >= w.rowptr[i]) and np.all(p < w.rowptr[i + 1])
        _same_bits(vals[p].astype(np.float64) * B[w.colind[p], j].astype(np.float64), c[i, j])


def pin_transposed_dense_and_scipy(O):
    """dB = A^T dC against the float64 dense product and scipy; mean scales each row by 1/len."""
    rp, ci, v = graphgen.random_csr(33, 29, 5.0, 71, empty_frac=0.15, duplicates=True, sort_cols=False)
    dC = graphgen.random_dense(33, 6, 72)
    rows = np.repeat(np.arange(33), np.diff(rp))
    lens = np.diff(rp).astype(np.float64)
    for op in ("sum", "mean"):
        for vv in (v, None):
            wts = (vv.astype(np.float64) if vv is not None else np.ones(len(ci)))
            if op == "mean":
                wts = wts / lens[rows]
            A = np.zeros((33, 29)); Aabs = np.zeros((33, 29))
            np.add.at(A, (rows, ci), wts)
            np.add.at(Aabs, (rows, ci), np.abs(wts))
            want = A.T @ dC.astype(np.float64)
            want_s = Aabs.T @ np.abs(dC.astype(np.float64))
            got, got_s = O.spmm_transposed(rp, ci, vv, dC, op, 29)
            _close(got, want, scale=want_s + 1e-30)
            _close(got_s, want_s)
    w = graphgen.workload(2, 0.02)
    dC = w.B(4)[: w.M]
    A = sp.csr_matrix((w.vals.astype(np.float64), w.colind, w.rowptr), shape=(w.M, w.K))
    got, got_s = O.spmm_transposed(w.rowptr, w.colind, w.vals, dC, "sum", w.K)
    _close(got, A.T @ dC.astype(np.float64), scale=got_s + 1e-30)


def pin_transposed_is_the_adjoint(O):
    """<A (x) B, dC> == <B, A^T (x) dC> for sum and for mean."""
    rp, ci, v = graphgen.random_csr(41, 37, 6.0, 81, empty_frac=0.1)
    B = graphgen.random_dense(37, 5, 81)
    dC = graphgen.random_dense(41, 5, 82)
    for op in ("sum", "mean"):
        C, S = O.spmm(rp, ci, v, B, op)
        dB, _ = O.spmm_transposed(rp, ci, v, dC, op, 37)
        lhs = float(np.sum(C * dC.astype(np.float64)))
        rhs = float(np.sum(B.astype(np.float64) * dB))
        assert abs(lhs - rhs) <= 1e-12 * float(np.sum(S * np.abs(dC))), (lhs, rhs)


def pin_pool_backward_numeric_gradient(O):
    """Routed gradient of max/min equals central differences of f(B) = sum(C(B) * dC) (piecewise linear)."""
    rng = np.random.default_rng(5)
    M, K, N = 9, 7, 3
    rp, ci, _ = graphgen.random_csr(M, K, 3.0, 91, empty_frac=0.2)
    v = rng.choice(np.array([1.0, -1.0, 2.0], dtype=np.float32), size=len(ci))
    dC = rng.integers(-4, 5, size=(M, N)).astype(np.float32)
    # integer-valued B with well separated products, so that +-h never changes which entry wins
    B = (rng.permutation(K * N).reshape(K, N) * 16 - 150).astype(np.float32)
    h = 0.25
    for op in ("max", "min"):
        C, arg = O.spmm_arg(rp, ci, v, B, op)
        for i in range(M):                                   # the margins the argument needs
            for j in range(N):
                prods = sorted(float(v[p]) * float(B[ci[p], j]) for p in range(rp[i], rp[i + 1]))
                assert all(b - a >= 4 for a, b in zip(prods, prods[1:]))
        dB, dS = O.pool_backward(ci, v, arg, dC, K)

        def f(Bx):
            c, _ = O.spmm(rp, ci, v, Bx, op)
            return float(np.sum(c * dC.astype(np.float64)))
        for k in range(K):
            for j in range(N):
                Bp, Bm = B.copy(), B.copy()
                Bp[k, j] += h
                Bm[k, j] -= h
                num = (f(Bp) - f(Bm)) / (2 * h)
                assert num == dB[k, j], (op, k, j, num, dB[k, j])
        assert np.all(dS >= np.abs(dB))
    # entry 0 is a legitimate position; -1 routes nothing
    arg = np.array([[0, -1]], dtype=np.int32)
    dB, _ = O.pool_backward(np.array([2], np.int32), np.array([3.0], np.float32), arg,
                            np.array([[5.0, 7.0]], np.float32), 4)
    want = np.zeros((4, 2)); want[2, 0] = 15.0
    _same_bits(dB, want)


def pin_csr_transpose(O):
    """Transposed CSR against scipy, as a permutation of the entries, and through the forward op."""
    rp, ci, v = graphgen.random_csr(45, 31, 5.0, 95, empty_frac=0.2, duplicates=True, sort_cols=False)
    rpT, ciT, vT = O.csr_transpose(rp, ci, v, 31)
    rows = np.repeat(np.arange(45), np.diff(rp))
    # every stored entry appears exactly once, under its column, rows of A ascending (stable)
    assert rpT[0] == 0 and rpT[-1] == len(ci) and np.array_equal(np.diff(rpT), np.bincount(ci, minlength=31))
    order = np.argsort(ci, kind="stable")
    assert np.array_equal(ciT, rows[order]) and np.array_equal(vT.view(np.uint32), v[order].view(np.uint32))
    A = sp.csr_matrix((v.astype(np.float64), ci, rp), shape=(45, 31))
    AT = sp.csr_matrix((vT.astype(np.float64), ciT, rpT), shape=(31, 45))
    assert abs(A.T - AT).max() < 1e-15
    # mean scaling: weights divided by the length of the entry's own row, rounded once to fp32
    _, _, vS = O.csr_transpose(rp, ci, v, 31, scale_by_row_length=True)
    lens = np.diff(rp).astype(np.float64)
    want = (v[order].astype(np.float64) / lens[rows[order]]).astype(np.float32)
    assert np.array_equal(vS.view(np.uint32), want.view(np.uint32))
    # vals == NULL stands for ones
    _, ciN, vN = O.csr_transpose(rp, ci, None, 31)
    assert np.array_equal(ciN, ciT) and (vN == 1).all()
    # the forward sum over the transposed arrays is the transposed product (gradient of sum / mean)
    dC = graphgen.random_dense(45, 4, 96)
    for scale, op in ((False, "sum"), (True, "mean")):
        rT, cT, wT = O.csr_transpose(rp, ci, v, 31, scale_by_row_length=scale)
        fwd, fs = O.spmm(rT, cT, wT, dC, "sum")
        ref, rs = O.spmm_transposed(rp, ci, v, dC, op, 31)
        _close(fwd, ref, scale=rs + 1e-30, tol=1e-7)       # the weights were rounded to fp32 once
    # empty matrix and trailing empty columns
    rT, cT, wT = O.csr_transpose(np.zeros(4, np.int32), np.zeros(0, np.int32), None, 6)
    assert not rT.any() and cT.size == 0


def pin_custom_fold(O):
    """The general fold with a user-supplied step: the built-in ops are special cases of it, and a
    fold that is none of them is checked against a per-entry Python loop."""
    rp, ci, v = graphgen.random_csr(25, 18, 4.0, 97, empty_frac=0.2, duplicates=True, sort_cols=False)
    B = graphgen.random_dense(18, 3, 97)
    for vv in (v, None):
        got = O.spmm_custom(rp, ci, vv, B, 0.0, lambda acc, a, b: acc + a * b)
        _same_bits(got, O.spmm(rp, ci, vv, B, "sum")[0])
        got = O.spmm_custom(rp, ci, vv, B, -math.inf, lambda acc, a, b: max(acc, a * b))
        _same_bits(got, O.spmm(rp, ci, vv, B, "max")[0])
        got = O.spmm_custom(rp, ci, vv, B, 0.0, lambda acc, a, b: acc + (a * b) ** 2)
        for i in range(25):
            for j in range(3):
                terms = [((float(vv[p]) if vv is not None else 1.0) * float(B[ci[p], j])) ** 2
                         for p in range(rp[i], rp[i + 1])]
                want = 0.0
                for t in terms:
                    want += t
                assert got[i, j] == want


GRAD_PINS = (pin_custom_fold, pin_csr_transpose, pin_arg_brute_force_with_ties, pin_arg_ties_inside_one_fp32_rounding_interval, pin_arg_consistent_with_forward, pin_transposed_dense_and_scipy,
             pin_transposed_is_the_adjoint, pin_pool_backward_numeric_gradient)
