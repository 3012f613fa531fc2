"""HyperLogLog reference in numpy / float64.  TEST INFRASTRUCTURE ONLY.

Follows the paper's Section 2.4 (sketch definition) and Section 3.1
(construct one sketch per row of B, merge by element-wise maximum along each
row of A, estimate from the merged sketch), with the estimator of the
HyperLogLog paper the text cites (Flajolet et al. 2007).  Shares no code with
the HIP sources; the hash below is restated here from its published
definition (the 32-bit finaliser of MurmurHash3).

Readings taken where the text leaves a choice:
  * register index = the low log2(m) bits of the 32-bit hash (Section 2.4:
    "lower hash bits");
  * register value = 1 + number of leading zeros of the remaining 32-log2(m)
    bits, 0 meaning "empty" (the standard rho of HyperLogLog, so that the
    standard bias constant alpha_m applies);
  * "harmonic mean + statistical correction" = alpha_m * m^2 / sum_j 2^-M[j],
    replaced by linear counting m*ln(m/V) when that raw value is <= 2.5 m and
    V > 0 registers are empty; no large-range correction (cardinalities here
    are far below 2^32 / 30);
  * one byte per register (Section 4.3).
"""
from __future__ import annotations

import numpy as np

_GOLDEN = np.uint32(0x9E3779B9)


def hash32(cols) -> np.ndarray:
    """MurmurHash3 fmix32 of (col + 0x9E3779B9) mod 2^32."""
    h = (np.asarray(cols).astype(np.uint64) + np.uint64(_GOLDEN)).astype(np.uint32)
    h = h ^ (h >> np.uint32(16))
    h = (h.astype(np.uint64) * np.uint64(0x85EBCA6B)).astype(np.uint32)
    h = h ^ (h >> np.uint32(13))
    h = (h.astype(np.uint64) * np.uint64(0xC2B2AE35)).astype(np.uint32)
    h = h ^ (h >> np.uint32(16))
    return h


def _log2(m: int) -> int:
    p = int(m).bit_length() - 1
    assert m >= 16 and (1 << p) == m, "m must be a power of two >= 16"
    return p


def index_and_rank(cols, m: int):
    """(register index, rank) of each column id."""
    p = _log2(m)
    h = hash32(cols)
    idx = (h & np.uint32(m - 1)).astype(np.int64)
    w = (h >> np.uint32(p)).astype(np.uint64)          # 32-p significant bits
    width = 32 - p
    # number of leading zeros of w inside `width` bits, +1; w == 0 -> width + 1
    bl = np.zeros(w.shape, dtype=np.int64)
    nz = w > 0
    bl[nz] = np.floor(np.log2(w[nz].astype(np.float64))).astype(np.int64) + 1  # bit length (exact below 2^53)
    rank = (width - bl + 1).astype(np.uint8)
    return idx, rank


def sketch(cols, m: int) -> np.ndarray:
    """m one-byte registers summarising the set of column ids."""
    reg = np.zeros(m, dtype=np.uint8)
    cols = np.asarray(cols)
    if cols.size:
        idx, rank = index_and_rank(cols, m)
        np.maximum.at(reg, idx, rank)
    return reg


def sketch_rows(B, m: int) -> np.ndarray:
    """One sketch per row of B: uint8 [B.rows, m] (Section 3.1, construct)."""
    S = np.zeros((B.rows, m), dtype=np.uint8)
    if B.nnz:
        idx, rank = index_and_rank(B.col_idx, m)
        row_of = np.repeat(np.arange(B.rows, dtype=np.int64), np.diff(B.row_ptr))
        np.maximum.at(S.reshape(-1), row_of * m + idx, rank)
    return S


def merge_rows(A, S_B: np.ndarray, rows=None) -> np.ndarray:
    """Merged sketch of each (selected) row of A: element-wise max over the
    sketches of the rows of B its entries point at (Section 3.1, merge)."""
    m = S_B.shape[1]
    rows = np.arange(A.rows) if rows is None else np.asarray(rows)
    out = np.zeros((len(rows), m), dtype=np.uint8)
    for t, i in enumerate(rows):
        ks = A.col_idx[A.row_ptr[i]:A.row_ptr[i + 1]]
        if ks.size:
            out[t] = S_B[ks].max(axis=0)
    return out


def alpha(m: int) -> float:
    if m == 16:
        return 0.673
    if m == 32:
        return 0.697
    if m == 64:
        return 0.709
    return 0.7213 / (1.0 + 1.079 / m)


def estimate(reg: np.ndarray) -> np.ndarray:
    """Cardinality estimate of each sketch (last axis = registers), float64."""
    reg = np.asarray(reg)
    m = reg.shape[-1]
    z = np.sum(np.ldexp(1.0, -reg.astype(np.int64)), axis=-1)
    raw = alpha(m) * m * m / z
    v = np.sum(reg == 0, axis=-1)
    with np.errstate(divide="ignore"):
        lin = m * np.log(m / np.maximum(v, 1).astype(np.float64))
    use_lin = (raw <= 2.5 * m) & (v > 0)
    return np.where(use_lin, lin, raw)


def estimate_rows(A, B, m: int, rows=None, prod=None, clamp: bool = True) -> np.ndarray:
    """Per-row estimate of nnz(C_i) via construct-and-merge.  With clamp=True
    the estimate is limited to what the structure already bounds exactly: at
    most min(prod[i], n) (Section 3.2: products are an upper bound) and at
    least the longest row of B the row touches."""
    S = sketch_rows(B, m)
    rows_arr = np.arange(A.rows) if rows is None else np.asarray(rows)
    est = estimate(merge_rows(A, S, rows_arr))
    if clamp:
        blen = np.diff(B.row_ptr)
        for t, i in enumerate(rows_arr):
            ks = A.col_idx[A.row_ptr[i]:A.row_ptr[i + 1]]
            lo = float(blen[ks].max()) if ks.size else 0.0
            hi = float(min(int(blen[ks].sum()), B.cols)) if ks.size else 0.0
            est[t] = min(max(est[t], lo), hi)
    return est
