"""The seeded input generators: shapes, counts and structure of each recipe.  CPU only."""
import numpy as np

from paper_2604_19004_amd import workloads as W


def _canonical(M):
    M.validate()
    for i in np.linspace(0, M.rows - 1, 50).astype(int):
        r = M.col_idx[M.row_ptr[i]:M.row_ptr[i + 1]]
        assert np.all(np.diff(r) > 0)


def test_er():
    A = W.erdos_renyi(4096, 8, seed=1)
    _canonical(A)
    assert np.all(np.diff(A.row_ptr) == 8) and np.all(np.abs(A.val) <= 1)
    assert np.array_equal(A.col_idx, W.erdos_renyi(4096, 8, seed=1).col_idx)
    d = np.diff(A.col_idx.reshape(4096, 8).astype(np.int64), axis=1)
    assert np.all(d > 0)


def test_laplacian():
    A = W.laplacian_2d(16)
    _canonical(A)
    assert A.nnz == 5 * 256 - 4 * 16
    rows = np.repeat(np.arange(A.rows), np.diff(A.row_ptr))
    assert np.all(A.val[rows == A.col_idx] == 4.0) and np.all(A.val[rows != A.col_idx] == -1.0)
    T = W.transpose(A)
    assert np.array_equal(T.col_idx, A.col_idx) and np.array_equal(T.val, A.val)   # symmetric


def test_rmat_small():
    A = W.rmat(10, 16, seed=3)
    _canonical(A)
    assert A.rows == 1024 and 0.4 * 16 * 1024 < A.nnz <= 16 * 1024   # duplicates merged
    deg = np.diff(A.row_ptr)
    assert deg.max() > 20 * max(1.0, np.median(deg))                     # heavy-tailed rows
    assert A.val.min() >= 0 and A.val.max() < 1
    # quadrant a (low row bits / low col bits) is the most likely: the first row/col half holds most entries
    rows = np.repeat(np.arange(A.rows), deg)
    assert np.mean(rows < 512) > 0.6 and np.mean(A.col_idx < 512) > 0.6


def test_rect_and_transpose():
    A = W.rect_poisson(4096, 1024, 8.0, seed=4)
    _canonical(A)
    deg = np.diff(A.row_ptr)
    assert abs(deg.mean() - 8.0) < 0.3 and deg.min() <= 2
    T = W.transpose(A)
    _canonical(T)
    assert (T.rows, T.cols, T.nnz) == (A.cols, A.rows, A.nnz)
    TT = W.transpose(T)
    assert np.array_equal(TT.row_ptr, A.row_ptr) and np.array_equal(TT.col_idx, A.col_idx) and np.array_equal(TT.val, A.val)


def test_clustered():
    A = W.clustered(16, 128, 0.2, 2, seed=5)
    _canonical(A)
    assert A.val.dtype == np.float32 and A.rows == 2048
    deg = np.diff(A.row_ptr)
    assert abs(deg.mean() - (0.2 * 128 + 2)) < 1.5
    colsum = np.bincount(A.col_idx, weights=A.val.astype(np.float64), minlength=A.cols)
    assert np.allclose(colsum[colsum > 0], 1.0, atol=1e-5)
    rows = np.repeat(np.arange(A.rows), deg)
    assert np.mean(rows // 128 == A.col_idx // 128) > 0.9
