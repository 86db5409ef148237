"""Matrix Market reader for user-supplied sparse matrices (e.g. files from the SuiteSparse
collection, which the paper's Section V-A draws its SNAP matrices from).  No such file ships
with this repository; this only turns a file the user has into the CSR arrays the library takes.
"""
from __future__ import annotations

import gzip

import numpy as np


def read_matrix_market(path):
    """Read a `coordinate` Matrix Market file (real, integer or pattern; general, symmetric or
    skew-symmetric).  Returns (M, K, rowptr int32, colind int32, vals float32) with the entries of
    every row sorted by column; repeated coordinates are kept as separate stored entries."""
    opener = gzip.open if str(path).endswith(".gz") else open
    with opener(path, "rt") as f:
        header = f.readline().strip().lower().split()
        if len(header) < 5 or header[0] != "%%matrixmarket" or header[1] != "matrix":
            raise ValueError("not a Matrix Market matrix file")
        layout, field, symmetry = header[2], header[3], header[4]
        if layout != "coordinate":
            raise ValueError("only the coordinate (sparse) layout is supported")
        if field not in ("real", "integer", "pattern"):
            raise ValueError(f"unsupported field '{field}'")
        if symmetry not in ("general", "symmetric", "skew-symmetric"):
            raise ValueError(f"unsupported symmetry '{symmetry}'")
        line = f.readline()
        while line.startswith("%") or not line.strip():
            line = f.readline()
        M, K, entries = (int(x) for x in line.split()[:3])
        cols = (0, 1) if field == "pattern" else (0, 1, 2)
        data = np.loadtxt(f, usecols=cols, ndmin=2, dtype=np.float64) if entries else np.zeros((0, len(cols)))
    if data.shape[0] != entries:
        raise ValueError(f"expected {entries} entries, found {data.shape[0]}")
    r = data[:, 0].astype(np.int64) - 1
    c = data[:, 1].astype(np.int64) - 1
    v = np.ones(entries) if field == "pattern" else data[:, 2]
    if entries and (r.min() < 0 or r.max() >= M or c.min() < 0 or c.max() >= K):
        raise ValueError("coordinate out of range")
    if symmetry != "general":
        off = r != c
        sign = -1.0 if symmetry == "skew-symmetric" else 1.0
        r, c, v = np.concatenate([r, c[off]]), np.concatenate([c, r[off]]), np.concatenate([v, sign * v[off]])
    order = np.lexsort((c, r))
    r, c, v = r[order], c[order], v[order]
    rowptr = np.zeros(M + 1, dtype=np.int64)
    np.cumsum(np.bincount(r, minlength=M), out=rowptr[1:])
    if rowptr[-1] >= 2**31:
        raise ValueError("too many entries for 32-bit indices")
    return M, K, rowptr.astype(np.int32), c.astype(np.int32), v.astype(np.float32)
