"""Seeded synthetic inputs (CSR graphs, edge values, dense feature matrices).

Inputs only: nothing here computes any part of SpMM.  The CPU oracle and the GPU
library are both fed from this module and share nothing else.

The five workloads below stand in for the paper's data (the citation graphs of
Table IV, the random graphs of Section V-B, the SNAP size/skew range of Section
V-A); the real dataset files are not used anywhere.
"""
from __future__ import annotations

import ctypes
import hashlib
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "graphgen.cpp")
_LIB = os.path.join(_HERE, "libgraphgen.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile graphgen.cpp into libgraphgen.so (g++, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O3", "-fopenmp", "-shared", "-fPIC", "-std=c++17", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    L = ctypes.CDLL(_LIB)
    i64, f64, u64, vp, ci = ctypes.c_int64, ctypes.c_double, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_int
    L.gg_csr_rows.restype = i64; L.gg_csr_rows.argtypes = [vp]
    L.gg_csr_cols.restype = i64; L.gg_csr_cols.argtypes = [vp]
    L.gg_csr_nnz.restype = i64; L.gg_csr_nnz.argtypes = [vp]
    L.gg_csr_copy.restype = None; L.gg_csr_copy.argtypes = [vp, vp, vp]
    L.gg_csr_free.restype = None; L.gg_csr_free.argtypes = [vp]
    L.gg_chung_lu_symmetric.restype = vp
    L.gg_chung_lu_symmetric.argtypes = [i64, f64, f64, i64, ci, u64]
    L.gg_chung_lu_directed.restype = vp
    L.gg_chung_lu_directed.argtypes = [i64, f64, f64, f64, i64, f64, u64]
    L.gg_rmat.restype = vp
    L.gg_rmat.argtypes = [i64, ci, f64, f64, f64, i64, f64, u64]
    L.gg_vals_sym_norm.restype = None; L.gg_vals_sym_norm.argtypes = [i64, vp, vp, vp]
    for name in ("gg_fill_uniform_01", "gg_fill_uniform_pm1", "gg_fill_normal"):
        fn = getattr(L, name)
        fn.restype = None
        fn.argtypes = [i64, u64, u64, vp]
    L.gg_max_threads.restype = ci
    L.gg_set_threads.restype = None; L.gg_set_threads.argtypes = [ci]
    _lib = L
    return L


def set_threads(n: int) -> None:
    _load().gg_set_threads(int(n))


def _take(handle):
    L = _load()
    if not handle:
        raise ValueError("graphgen: invalid generator arguments")
    try:
        M, K, nnz = L.gg_csr_rows(handle), L.gg_csr_cols(handle), L.gg_csr_nnz(handle)
        rowptr = np.empty(M + 1, dtype=np.int32)
        colind = np.empty(nnz, dtype=np.int32)
        L.gg_csr_copy(handle, rowptr.ctypes.data, colind.ctypes.data)
    finally:
        L.gg_csr_free(handle)
    return int(M), int(K), rowptr, colind


def chung_lu_symmetric(M, edges, seed, gamma=2.5, max_over_mean=40.0, exact=False):
    return _take(_load().gg_chung_lu_symmetric(M, gamma, max_over_mean, edges, int(exact), seed))


def chung_lu_directed(M, edges, seed, gamma=2.5, max_over_mean_out=70.0, max_over_mean_in=70.0,
                      empty_frac=0.0):
    return _take(_load().gg_chung_lu_directed(M, gamma, max_over_mean_out, max_over_mean_in,
                                              edges, empty_frac, seed))


def rmat(M, scale, draws, seed, a=0.57, b=0.19, c=0.19, extra_empty_frac=0.0):
    return _take(_load().gg_rmat(M, scale, a, b, c, draws, extra_empty_frac, seed))


def vals_sym_norm(rowptr, colind):
    vals = np.empty(colind.shape[0], dtype=np.float32)
    _load().gg_vals_sym_norm(rowptr.shape[0] - 1, rowptr.ctypes.data, colind.ctypes.data,
                             vals.ctypes.data)
    return vals


def _fill(name, shape, seed, stream):
    out = np.empty(shape, dtype=np.float32)
    getattr(_load(), name)(out.size, seed, stream, out.ctypes.data)
    return out


def uniform_01(shape, seed, stream=0):
    """fp32 uniform on (0, 1]."""
    return _fill("gg_fill_uniform_01", shape, seed, stream)


def uniform_pm1(shape, seed, stream=0):
    """fp32 uniform on (-1, 1), never exactly zero."""
    return _fill("gg_fill_uniform_pm1", shape, seed, stream)


def normal(shape, seed, stream=0):
    """fp32 standard normal, never exactly zero."""
    return _fill("gg_fill_normal", shape, seed, stream)


# --------------------------------------------------------------------------
# The five workloads
# --------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    M: int
    K: int
    rowptr: np.ndarray
    colind: np.ndarray
    vals: np.ndarray | None
    seed: int
    b_kind: str                       # "uniform_pm1" | "normal"
    widths: tuple                     # feature widths N this workload is run at
    ops: tuple                        # reduce ops this workload is run with
    meta: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.colind.shape[0])

    def B(self, N: int) -> np.ndarray:
        fill = uniform_pm1 if self.b_kind == "uniform_pm1" else normal
        return fill((self.K, N), self.seed, stream=N)

    def describe(self) -> dict:
        lens = np.diff(self.rowptr)
        h = hashlib.blake2b(digest_size=8)
        h.update(self.rowptr.tobytes()); h.update(self.colind.tobytes())
        return {"name": self.name, "M": self.M, "K": self.K, "nnz": self.nnz,
                "max_row": int(lens.max()) if self.M else 0,
                "mean_row": float(lens.mean()) if self.M else 0.0,
                "empty_rows": float((lens == 0).mean()) if self.M else 0.0,
                "csr_hash": h.hexdigest(), **self.meta}


WORKLOAD_NAMES = ("tiny_citation", "width_sweep", "general_ops", "large_dense_degree", "skew_narrow")
# extra shapes: the uniform random graphs of the paper's Section V-B (Tables V and VI), N = 512
EXTRA_WORKLOAD_NAMES = ("uniform_random_65k", "uniform_random_262k")

# number of Chung-Lu candidate pairs for "large_dense_degree": hub-hub pairs repeat
# and are merged, so more than 114.6M/2 candidates are needed to land near 114.6M nnz
_LARGE_CANDIDATES = 58_170_000


def workload(which, scale: float = 1.0) -> Workload:
    """Build workload `which` (index 0..4 or a name from WORKLOAD_NAMES).

    `scale` < 1 shrinks M and the edge budget proportionally (used by CPU tests
    and by quick parity runs); scale == 1 is the full size.
    """
    s = float(scale)
    if which in EXTRA_WORKLOAD_NAMES:
        log2m, draws = (16, 650_000) if which == "uniform_random_65k" else (18, 2_600_000)
        M = max(8, int(round((1 << log2m) * s)))
        sc = max(3, int(np.ceil(np.log2(M))))
        M, K, rp, ci = rmat(M, sc, int(round(draws * s)), seed=10 + log2m, a=0.25, b=0.25, c=0.25)
        return Workload(which, M, K, rp, ci, uniform_01(ci.shape[0], 10 + log2m), 10 + log2m,
                        "uniform_pm1", (512,), ("sum", "max"))
    idx = WORKLOAD_NAMES.index(which) if isinstance(which, str) else int(which)
    name = WORKLOAD_NAMES[idx]
    if idx == 0:
        M = max(8, int(round(2708 * s)))
        e = max(4, int(round(5278 * s)))
        M, K, rp, ci = chung_lu_symmetric(M, e, seed=0, max_over_mean=40.0, exact=True)
        return Workload(name, M, K, rp, ci, vals_sym_norm(rp, ci), 0, "uniform_pm1", (16,), ("sum",))
    if idx == 1:
        M = max(8, int(round(19717 * s)))
        e = max(4, int(round(44324 * s)))
        M, K, rp, ci = chung_lu_symmetric(M, e, seed=1, max_over_mean=40.0, exact=True)
        return Workload(name, M, K, rp, ci, uniform_01(ci.shape[0], 1), 1, "uniform_pm1",
                        (32, 64, 128, 256, 512), ("sum",))
    if idx == 2:
        M = max(8, int(round(169343 * s)))
        e = int(round(2_402_500 * s))
        M, K, rp, ci = chung_lu_directed(M, e, seed=2, empty_frac=0.03)
        return Workload(name, M, K, rp, ci, np.ones(ci.shape[0], dtype=np.float32), 2, "normal",
                        (128,), ("sum", "mean", "max", "min"))
    if idx == 3:
        M = max(8, int(round(232965 * s)))
        e = int(round(_LARGE_CANDIDATES * s))
        # M and the candidate budget shrink together, so the mean degree stays near 492
        M, K, rp, ci = chung_lu_symmetric(M, e, seed=3, max_over_mean=40.6, exact=False)
        return Workload(name, M, K, rp, ci, vals_sym_norm(rp, ci), 3, "uniform_pm1", (64,),
                        ("sum", "max"))
    if idx == 4:
        M = max(8, int(round(1_000_000 * s)))
        sc = max(3, int(np.ceil(np.log2(M))))
        draws = int(round(16_000_000 * s))
        M, K, rp, ci = rmat(M, sc, draws, seed=4)
        empty = float((np.diff(rp) == 0).mean())
        if empty < 0.05:  # top up to 5 % empty rows only when R-MAT left fewer on its own
            M, K, rp, ci = rmat(M, sc, draws, seed=4, extra_empty_frac=0.05 - empty)
        return Workload(name, M, K, rp, ci, uniform_01(ci.shape[0], 4), 4, "uniform_pm1", (8, 32),
                        ("sum", "mean"), {"rmat_scale": sc})
    raise ValueError(which)


def workload_from_matrix_market(path, widths=(128, 256, 512), seed=100) -> Workload:
    """A user-supplied Matrix Market file (e.g. from SuiteSparse) as a workload; the feature
    matrix is seeded uniform(-1, 1) and the stored values are the file's."""
    from .mtx import read_matrix_market
    M, K, rp, ci, v = read_matrix_market(path)
    return Workload(os.path.basename(str(path)), M, K, rp, ci, v, seed, "uniform_pm1", tuple(widths),
                    ("sum", "max"), {"source": "matrix market file"})


# --------------------------------------------------------------------------
# A suite of matrix shapes standing in for the range of a sparse-matrix collection
# (Section V-A evaluates on many collection matrices and reports geometric means,
# Table VII).  Every matrix is generated here from a seed; none is a collection file.
# --------------------------------------------------------------------------
def _csr_from_offsets(dims, offsets):
    """Stencil on a regular grid of shape `dims`: vertex x is joined to x + o for every offset
    vector o that stays inside the grid (no wrap-around).  Rows come out with sorted columns."""
    dims = tuple(int(d) for d in dims)
    M = int(np.prod(dims))
    coords = np.unravel_index(np.arange(M, dtype=np.int64), dims)
    strides = [int(np.prod(dims[a + 1:])) for a in range(len(dims))]
    offsets = sorted(offsets, key=lambda o: sum(x * st for x, st in zip(o, strides)))
    cols = np.full((M, len(offsets)), -1, dtype=np.int64)
    for t, o in enumerate(offsets):
        ok = np.ones(M, dtype=bool)
        for a, d in enumerate(dims):
            ok &= (coords[a] + o[a] >= 0) & (coords[a] + o[a] < d)
        cols[ok, t] = np.arange(M, dtype=np.int64)[ok] + sum(x * st for x, st in zip(o, strides))
    keep = cols >= 0
    rowptr = np.zeros(M + 1, dtype=np.int64)
    np.cumsum(keep.sum(axis=1), out=rowptr[1:])
    return M, M, rowptr.astype(np.int32), cols[keep].astype(np.int32)


def grid2d(n):
    """5-point stencil on an n x n grid (mesh / road-network-like: short rows, banded)."""
    return _csr_from_offsets((n, n), [(0, 0), (0, 1), (0, -1), (1, 0), (-1, 0)])


def grid3d(n):
    """27-point stencil on an n^3 grid (finite-element-like: equal rows of up to 27 entries)."""
    offs = [(a, b, c) for a in (-1, 0, 1) for b in (-1, 0, 1) for c in (-1, 0, 1)]
    return _csr_from_offsets((n, n, n), offs)


SUITE = {
    # name: (builder, seed); M, entries and degree structure span a few 10^4 .. 10^6 rows,
    # mean row length 3 .. 130, flat / power-law / R-MAT-skewed / banded
    "powerlaw_30k_d8":    (lambda: chung_lu_symmetric(30_000, 120_000, seed=201, max_over_mean=30.0), 201),
    "powerlaw_100k_d30":  (lambda: chung_lu_symmetric(100_000, 1_500_000, seed=202, max_over_mean=60.0), 202),
    "powerlaw_400k_d10":  (lambda: chung_lu_symmetric(400_000, 2_000_000, seed=203, max_over_mean=200.0), 203),
    "powerlaw_1m_d6":     (lambda: chung_lu_symmetric(1_000_000, 3_000_000, seed=204, max_over_mean=400.0), 204),
    "web_200k_d20":       (lambda: chung_lu_directed(200_000, 4_000_000, seed=205, max_over_mean_out=40.0,
                                                     max_over_mean_in=400.0), 205),
    "web_800k_d6":        (lambda: chung_lu_directed(800_000, 4_800_000, seed=206, max_over_mean_out=100.0,
                                                     max_over_mean_in=1000.0, empty_frac=0.1), 206),
    "rmat_64k_d16":       (lambda: rmat(1 << 16, 16, 1 << 20, seed=207), 207),
    "rmat_256k_d16":      (lambda: rmat(1 << 18, 18, 1 << 22, seed=208), 208),
    "rmat_1m_d8":         (lambda: rmat(1 << 20, 20, 1 << 23, seed=209), 209),
    "uniform_128k_d10":   (lambda: rmat(1 << 17, 17, 1_310_000, seed=210, a=0.25, b=0.25, c=0.25), 210),
    "uniform_512k_d4":    (lambda: rmat(1 << 19, 19, 2_100_000, seed=211, a=0.25, b=0.25, c=0.25), 211),
    "dense_rows_40k_d130": (lambda: chung_lu_symmetric(40_000, 2_600_000, seed=212, max_over_mean=10.0), 212),
    "grid2d_1000":        (lambda: grid2d(1000), 213),
    "grid2d_300":         (lambda: grid2d(300), 214),
    "grid3d_64":          (lambda: grid3d(64), 215),
    "grid3d_100":         (lambda: grid3d(100), 216),
}
SUITE_NAMES = tuple(SUITE)


def suite_matrix(name) -> Workload:
    """One matrix of the shape suite, values uniform(0, 1], run at N = 128 / 256 / 512 as in Table VII."""
    builder, seed = SUITE[name]
    M, K, rp, ci = builder()
    return Workload(name, M, K, rp, ci, uniform_01(ci.shape[0], seed), seed, "uniform_pm1",
                    (128, 256, 512), ("sum",), {"source": "shape suite"})


# --------------------------------------------------------------------------
# Small random CSR matrices for unit tests (numpy's seeded PCG64)
# --------------------------------------------------------------------------
def random_csr(M, K, mean_len, seed, empty_frac=0.0, duplicates=False, sort_cols=True,
               long_rows=(), val_kind="uniform"):
    """Random CSR with geometric-ish row lengths.

    long_rows: iterable of (row, length) forcing specific long rows.
    duplicates=True draws columns with replacement (repeated column indices stay as
    separate stored entries); sort_cols=False leaves the columns in draw order.
    """
    rng = np.random.default_rng(seed)
    lens = rng.geometric(1.0 / max(mean_len, 1.0), size=M).astype(np.int64) if M else np.zeros(0, np.int64)
    if not duplicates:
        lens = np.minimum(lens, K)
    if empty_frac > 0 and M:
        lens[rng.random(M) < empty_frac] = 0
    for r, ln in long_rows:
        lens[r] = ln if duplicates else min(ln, K)
    if K == 0:
        lens[:] = 0
    rowptr = np.zeros(M + 1, dtype=np.int64)
    np.cumsum(lens, out=rowptr[1:])
    nnz = int(rowptr[-1])
    colind = np.empty(nnz, dtype=np.int32)
    for i in range(M):
        n = int(lens[i])
        if n == 0:
            continue
        if duplicates:
            c = rng.integers(0, K, size=n)
        elif n * 4 > K:
            c = rng.permutation(K)[:n]
        else:
            c = np.unique(rng.integers(0, K, size=2 * n + 8))
            while c.shape[0] < n:
                c = np.unique(np.concatenate([c, rng.integers(0, K, size=2 * n + 8)]))
            c = rng.permutation(c)[:n]
        colind[rowptr[i]:rowptr[i + 1]] = np.sort(c) if sort_cols else c
    if val_kind == "uniform":
        vals = (rng.random(nnz) * 2.0 - 1.0).astype(np.float32)
    elif val_kind == "ones":
        vals = np.ones(nnz, dtype=np.float32)
    else:
        raise ValueError(val_kind)
    return rowptr.astype(np.int32), colind, vals


def random_dense(K, N, seed):
    rng = np.random.default_rng(seed + 0x5EED)
    return (rng.random((K, N)) * 2.0 - 1.0).astype(np.float32)
