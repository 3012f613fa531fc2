"""Seeded synthetic CSR inputs for SpGEMM (C = A*B).

This module only *generates inputs*.  It contains none of the method's
arithmetic (no products, no sketches, no accumulation) so that the CPU
checker and the HIP path can both consume exactly the same arrays while
sharing no code of their own.

Every generator returns a :class:`CSR` with ``row_ptr`` (int64, rows+1),
``col_idx`` (int32, ascending inside each row, no duplicates) and ``val``
(float64 or float32).  The five named workloads stand in for the matrix
collections the paper evaluates on (square matrices for C = A*A and
rectangular ones for C = A*A^T, Section 5.1): a smoke-size random matrix, a
stencil (AMG-like) matrix, a power-law graph, a rectangular overlap product
and a Markov-clustering expansion step.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class CSR:
    rows: int
    cols: int
    row_ptr: np.ndarray  # int64 [rows+1]
    col_idx: np.ndarray  # int32 [nnz]
    val: np.ndarray      # float64 / float32 [nnz]

    @property
    def nnz(self) -> int:
        return int(self.row_ptr[-1])

    def validate(self) -> None:
        rp, ci = self.row_ptr, self.col_idx
        assert rp.dtype == np.int64 and ci.dtype == np.int32
        assert rp.shape == (self.rows + 1,) and rp[0] == 0
        assert np.all(np.diff(rp) >= 0)
        assert ci.shape == (rp[-1],) and self.val.shape == (rp[-1],)
        if ci.size:
            assert ci.min() >= 0 and ci.max() < self.cols


def _from_sorted_keys(rows: int, cols: int, key: np.ndarray, val_fn) -> CSR:
    """key = row * cols + col, already unique and ascending."""
    r = (key // cols).astype(np.int64)
    c = (key % cols).astype(np.int32)
    counts = np.bincount(r, minlength=rows).astype(np.int64)
    rp = np.zeros(rows + 1, dtype=np.int64)
    np.cumsum(counts, out=rp[1:])
    return CSR(rows, cols, rp, c, val_fn(key.size))


def from_coo(rows: int, cols: int, r: np.ndarray, c: np.ndarray, val_fn) -> CSR:
    """Merge duplicate (r, c) pairs into one entry, sort, build CSR."""
    key = np.unique(r.astype(np.int64) * np.int64(cols) + c.astype(np.int64))
    return _from_sorted_keys(rows, cols, key, val_fn)


def transpose(a: CSR) -> CSR:
    """Explicit CSR of A^T (input preparation for the C = A*A^T workloads)."""
    nnz = a.nnz
    row_of = np.repeat(np.arange(a.rows, dtype=np.int64), np.diff(a.row_ptr))
    order = np.argsort(a.col_idx.astype(np.int64) * np.int64(a.rows) + row_of, kind="stable")
    counts = np.bincount(a.col_idx, minlength=a.cols).astype(np.int64)
    rp = np.zeros(a.cols + 1, dtype=np.int64)
    np.cumsum(counts, out=rp[1:])
    assert rp[-1] == nnz
    return CSR(a.cols, a.rows, rp, row_of[order].astype(np.int32), a.val[order].copy())


# --------------------------------------------------------------------------
# 1. Erdos-Renyi-like: exactly `per_row` distinct uniform columns per row.
# --------------------------------------------------------------------------
def erdos_renyi(n: int = 4096, per_row: int = 8, seed: int = 1, cols: int | None = None) -> CSR:
    cols = n if cols is None else cols
    assert per_row <= cols
    rng = np.random.default_rng(seed)
    c = rng.integers(0, cols, size=(n, per_row), dtype=np.int64)
    c.sort(axis=1)
    while True:  # redraw rows that contain a repeated column
        bad = np.nonzero((np.diff(c, axis=1) == 0).any(axis=1))[0]
        if bad.size == 0:
            break
        c[bad] = np.sort(rng.integers(0, cols, size=(bad.size, per_row), dtype=np.int64), axis=1)
    rp = np.arange(n + 1, dtype=np.int64) * per_row
    val = rng.uniform(-1.0, 1.0, size=n * per_row)
    return CSR(n, cols, rp, c.reshape(-1).astype(np.int32), val)


# --------------------------------------------------------------------------
# 2. 2-D five-point Laplacian on a g x g grid (diag 4, off-diag -1).
# --------------------------------------------------------------------------
def laplacian_2d(g: int = 1024) -> CSR:
    n = g * g
    idx = np.arange(n, dtype=np.int64)
    x, y = idx % g, idx // g
    # neighbours in ascending column order: (y-1), (x-1), self, (x+1), (y+1)
    cand = np.stack([idx - g, idx - 1, idx, idx + 1, idx + g], axis=1)
    ok = np.stack([y > 0, x > 0, np.ones(n, bool), x < g - 1, y < g - 1], axis=1)
    v = np.broadcast_to(np.array([-1.0, -1.0, 4.0, -1.0, -1.0]), (n, 5))
    rp = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(ok.sum(axis=1), out=rp[1:])
    return CSR(n, n, rp, cand[ok].astype(np.int32), v[ok].astype(np.float64).copy())


# --------------------------------------------------------------------------
# 3. R-MAT (recursive quadrant choice per bit level), duplicates merged.
# --------------------------------------------------------------------------
def rmat(scale: int = 20, edge_factor: int = 16, abcd=(0.57, 0.19, 0.19, 0.05), seed: int = 3,
         chunk: int = 1 << 22) -> CSR:
    n = 1 << scale
    n_edges = edge_factor * n
    a, b, c, _d = abcd
    rng = np.random.default_rng(seed)
    keys = []
    for start in range(0, n_edges, chunk):
        cnt = min(chunk, n_edges - start)
        r = np.zeros(cnt, dtype=np.int64)
        cc = np.zeros(cnt, dtype=np.int64)
        for _level in range(scale):
            u = rng.random(cnt)
            # quadrant a: (0,0)  b: (0,1)  c: (1,0)  d: (1,1)
            rbit = u >= a + b
            cbit = ((u >= a) & (u < a + b)) | (u >= a + b + c)
            r = (r << 1) | rbit
            cc = (cc << 1) | cbit
        keys.append(r * np.int64(n) + cc)
    key = np.unique(np.concatenate(keys))
    return _from_sorted_keys(n, n, key, lambda k: rng.uniform(0.0, 1.0, size=k))


# --------------------------------------------------------------------------
# 4. Rectangular, Poisson(lam) entries per row at uniform columns.
# --------------------------------------------------------------------------
def rect_poisson(rows: int = 524288, cols: int = 131072, lam: float = 8.0, seed: int = 4) -> CSR:
    rng = np.random.default_rng(seed)
    cnt = rng.poisson(lam, size=rows).astype(np.int64)
    r = np.repeat(np.arange(rows, dtype=np.int64), cnt)
    c = rng.integers(0, cols, size=r.size, dtype=np.int64)
    return from_coo(rows, cols, r, c, lambda k: rng.uniform(-1.0, 1.0, size=k))


# --------------------------------------------------------------------------
# 5. Clustered graph: communities of `size` nodes, dense-ish inside, a few
#    random links outside, float32 values made column-stochastic.
#    Every ordered pair inside a community, the diagonal included, is kept
#    with probability `density`.
# --------------------------------------------------------------------------
def clustered(communities: int = 4096, size: int = 128, density: float = 0.2, inter: int = 2,
              seed: int = 5) -> CSR:
    n = communities * size
    rng = np.random.default_rng(seed)
    keys = []
    block = 256  # communities per batch keeps the Bernoulli mask small
    for c0 in range(0, communities, block):
        nb = min(block, communities - c0)
        mask = rng.random((nb, size, size)) < density
        cb, ri, ci = np.nonzero(mask)
        base = (cb.astype(np.int64) + c0) * size
        keys.append((base + ri) * np.int64(n) + base + ci)
    r = np.repeat(np.arange(n, dtype=np.int64), inter)
    c = rng.integers(0, n, size=r.size, dtype=np.int64)
    keys.append(r * np.int64(n) + c)
    key = np.unique(np.concatenate(keys))
    m = _from_sorted_keys(n, n, key, lambda k: rng.uniform(0.0, 1.0, size=k))
    colsum = np.bincount(m.col_idx, weights=m.val, minlength=n)
    m.val = (m.val / colsum[m.col_idx]).astype(np.float32)
    return m


# --------------------------------------------------------------------------
# Named workloads: (A, B) pairs for C = A*B.
# --------------------------------------------------------------------------
WORKLOADS = ("er", "laplacian", "rmat", "rect", "clustered")


def make(name: str, small: bool = False):
    """Return (A, B, description).  ``small=True`` shrinks the instance (same
    recipe, same structure) to something a CPU checks in about a second."""
    if name == "er":
        a = erdos_renyi(4096, 8, seed=1)
        return a, a, "Erdos-Renyi 4096x4096, 8 distinct columns/row, fp64 U(-1,1), C=A*A"
    if name == "laplacian":
        g = 96 if small else 1024
        a = laplacian_2d(g)
        return a, a, f"2-D 5-point Laplacian {g}x{g} grid, fp64, C=A*A"
    if name == "rmat":
        s = 12 if small else 20
        a = rmat(s, 16, seed=3)
        return a, a, f"R-MAT scale {s}, edge factor 16, (0.57,0.19,0.19,0.05), fp64 U(0,1), C=A*A"
    if name == "rect":
        r, c = (8192, 2048) if small else (524288, 131072)
        a = rect_poisson(r, c, 8.0, seed=4)
        return a, transpose(a), f"rectangular {r}x{c}, Poisson(8)/row, fp64 U(-1,1), C=A*A^T"
    if name == "clustered":
        k = 64 if small else 4096
        a = clustered(k, 128, 0.2, 2, seed=5)
        return a, a, f"clustered {k} communities x 128, density 0.2 + 2 random links, fp32 column-stochastic, C=A*A"
    raise ValueError(f"unknown workload {name!r}; choose from {WORKLOADS}")
