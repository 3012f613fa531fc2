"""ctypes front end of the C oracle (``ocean_oracle.c``).  TEST INFRASTRUCTURE ONLY.

The arithmetic lives in the C file; this module only marshals numpy arrays,
walks row blocks and assembles CSR results.  See the C file's header for what
is computed and which passages of the paper define it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ocean_oracle.c")
_LIB = os.path.join(_HERE, "libocean_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the C oracle with gcc (OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        i64, p = ctypes.c_int64, ctypes.c_void_p
        lib.oracle_row_products.restype = i64
        lib.oracle_row_products.argtypes = [i64, p, p, p, p]
        lib.oracle_count_rows.restype = None
        lib.oracle_count_rows.argtypes = [i64, i64, p, p, p, p, i64, p]
        lib.oracle_multiply_rows.restype = None
        lib.oracle_multiply_rows.argtypes = [i64, i64, p, p, p, p, p, p, i64, p, p, p, p]
        lib.oracle_set_threads.argtypes = [ctypes.c_int]
        lib.oracle_get_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def set_threads(t: int) -> None:
    _load().oracle_set_threads(int(t))


def get_threads() -> int:
    return int(_load().oracle_get_threads())


def _ptr(a: np.ndarray) -> int:
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data


def _chk(A, B):
    assert A.cols == B.rows, "inner dimensions differ"
    for M in (A, B):
        assert M.row_ptr.dtype == np.int64 and M.col_idx.dtype == np.int32


def row_products(A, B) -> np.ndarray:
    """prod[i] = number of intermediate products of row i (int64)."""
    _chk(A, B)
    prod = np.zeros(A.rows, dtype=np.int64)
    total = _load().oracle_row_products(A.rows, _ptr(A.row_ptr), _ptr(A.col_idx), _ptr(B.row_ptr), _ptr(prod))
    assert total == int(prod.sum())
    return prod


def count_rows(A, B, r0: int = 0, r1: int | None = None) -> np.ndarray:
    """Exact nnz of rows [r0, r1) of C (int64)."""
    _chk(A, B)
    r1 = A.rows if r1 is None else r1
    nnz = np.zeros(max(r1 - r0, 0), dtype=np.int64)
    if r1 > r0:
        _load().oracle_count_rows(r0, r1, _ptr(A.row_ptr), _ptr(A.col_idx), _ptr(B.row_ptr), _ptr(B.col_idx),
                                  B.cols, _ptr(nnz))
    return nnz


@dataclass
class RowBlock:
    r0: int
    r1: int
    row_ptr: np.ndarray   # int64 [r1-r0+1], relative to the block
    col_idx: np.ndarray   # int32
    val: np.ndarray       # float64
    absval: np.ndarray    # float64, sum_k |A_ik*B_kj|


def multiply_rows(A, B, r0: int = 0, r1: int | None = None, nnz: np.ndarray | None = None) -> RowBlock:
    """Rows [r0, r1) of C = A*B: structure, values and per-entry |.| sums, all in double.
    nnz: the result of count_rows(A, B, r0, r1) when the caller already holds it (saves the recount)."""
    _chk(A, B)
    r1 = A.rows if r1 is None else r1
    if nnz is None:
        nnz = count_rows(A, B, r0, r1)
    assert len(nnz) == max(r1 - r0, 0)
    rp = np.zeros(len(nnz) + 1, dtype=np.int64)
    np.cumsum(nnz, out=rp[1:])
    tot = int(rp[-1])
    col = np.zeros(tot, dtype=np.int32)
    val = np.zeros(tot, dtype=np.float64)
    ab = np.zeros(tot, dtype=np.float64)
    if r1 > r0:
        av = np.ascontiguousarray(A.val, dtype=np.float64)
        bv = av if B is A else np.ascontiguousarray(B.val, dtype=np.float64)
        _load().oracle_multiply_rows(r0, r1, _ptr(A.row_ptr), _ptr(A.col_idx), _ptr(av), _ptr(B.row_ptr),
                                     _ptr(B.col_idx), _ptr(bv), B.cols, _ptr(rp), _ptr(col), _ptr(val), _ptr(ab))
    return RowBlock(r0, r1, rp, col, val, ab)


def multiply_row_list(A, B, rows) -> list:
    """One RowBlock per requested row index (for sampled checks of very large products)."""
    return [multiply_rows(A, B, int(r), int(r) + 1) for r in rows]
