"""Pins for the CPU SpGEMM oracle (oracle/ocean_oracle.c) against things other
than itself: brute-force dense products, closed forms, structural invariants,
algebraic identities and SciPy as an independent black box.  CPU only."""
import numpy as np
import pytest
import scipy.sparse as sp

from oracle import spgemm as O
from paper_2604_19004_amd import workloads as W
from paper_2604_19004_amd.workloads import CSR


def csr_from_dense_pattern(vals: np.ndarray, pattern: np.ndarray) -> CSR:
    """CSR that stores exactly the entries where pattern is True (values may be 0.0)."""
    rows, cols = vals.shape
    rp = np.zeros(rows + 1, dtype=np.int64)
    np.cumsum(pattern.sum(axis=1), out=rp[1:])
    r, c = np.nonzero(pattern)
    return CSR(rows, cols, rp, c.astype(np.int32), vals[r, c].astype(np.float64))


def brute(A_vals, A_pat, B_vals, B_pat):
    """Dense definition: values by dense matmul of the stored entries, structure from
    the boolean product of the patterns (never from value != 0)."""
    Cv = (A_vals * A_pat) @ (B_vals * B_pat)
    Cabs = (np.abs(A_vals) * A_pat) @ (np.abs(B_vals) * B_pat)
    Cp = (A_pat.astype(np.int64) @ B_pat.astype(np.int64)) > 0
    return Cv, Cabs, Cp


def check_against_brute(A_vals, A_pat, B_vals, B_pat):
    A = csr_from_dense_pattern(A_vals, A_pat)
    B = csr_from_dense_pattern(B_vals, B_pat)
    blk = O.multiply_rows(A, B)
    Cv, Cabs, Cp = brute(A_vals, A_pat, B_vals, B_pat)
    rows, n = Cp.shape
    assert np.array_equal(np.diff(blk.row_ptr), Cp.sum(axis=1))
    for i in range(rows):
        s, e = blk.row_ptr[i], blk.row_ptr[i + 1]
        want = np.nonzero(Cp[i])[0]
        assert np.array_equal(blk.col_idx[s:e], want)          # ascending, exact structure
        np.testing.assert_allclose(blk.val[s:e], Cv[i, want], rtol=0, atol=1e-13 * (1 + Cabs[i, want].max(initial=0)))
        np.testing.assert_allclose(blk.absval[s:e], Cabs[i, want], rtol=1e-14, atol=0)
    assert np.array_equal(O.count_rows(A, B), Cp.sum(axis=1))
    assert np.array_equal(O.row_products(A, B), (A_pat.astype(np.int64) @ B_pat.sum(axis=1).astype(np.int64)))


@pytest.mark.parametrize("seed", range(12))
def test_brute_force_random_rectangular(seed):
    rng = np.random.default_rng(seed)
    m, k, n = rng.integers(1, 40, size=3)
    dens = rng.choice([0.05, 0.2, 0.6])
    A_pat = rng.random((m, k)) < dens
    B_pat = rng.random((k, n)) < dens
    # a few empty rows / columns on purpose
    if m > 2:
        A_pat[rng.integers(m)] = False
    if k > 2:
        B_pat[rng.integers(k)] = False
        A_pat[:, rng.integers(k)] = False
    A_vals = rng.uniform(-1, 1, (m, k))
    B_vals = rng.uniform(-1, 1, (k, n))
    check_against_brute(A_vals, A_pat, B_vals, B_pat)


def test_brute_force_special_cases():
    one = np.ones((1, 1))
    check_against_brute(3.0 * one, one > 0, -2.0 * one, one > 0)                # 1x1
    check_against_brute(one, one < 0, one, one > 0)                              # 1x1, A empty
    # a row that reaches every column, through a full row of B
    A_pat = np.zeros((3, 4), bool); A_pat[1, 2] = True
    B_pat = np.zeros((4, 9), bool); B_pat[2, :] = True
    check_against_brute(np.full((3, 4), 0.5), A_pat, np.arange(36.).reshape(4, 9), B_pat)
    # explicit zeros are structural: stored 0.0 in A still produces entries
    A_pat = np.array([[True, True], [False, True]])
    A_vals = np.array([[0.0, 2.0], [0.0, 0.0]])
    B_pat = np.array([[True, False, True], [False, True, False]])
    B_vals = np.array([[1.0, 0.0, 5.0], [0.0, 0.0, 0.0]])
    check_against_brute(A_vals, A_pat, B_vals, B_pat)


def test_exact_cancellation_is_kept_as_stored_zero():
    # C_00 = (+1)(1) + (-1)(1) = 0 but the entry must exist
    A = CSR(1, 2, np.array([0, 2], np.int64), np.array([0, 1], np.int32), np.array([1.0, -1.0]))
    B = CSR(2, 3, np.array([0, 1, 3], np.int64), np.array([0, 0, 2], np.int32), np.array([1.0, 1.0, 7.0]))
    blk = O.multiply_rows(A, B)
    assert blk.col_idx.tolist() == [0, 2]
    assert blk.val.tolist() == [0.0, -7.0]
    assert blk.absval.tolist() == [2.0, 7.0]


def test_duplicate_and_unsorted_inputs_add_terms():
    # row 0 of A stores column 1 twice, B's row 1 is unsorted with a repeated column
    A = CSR(1, 2, np.array([0, 2], np.int64), np.array([1, 1], np.int32), np.array([2.0, 3.0]))
    B = CSR(2, 4, np.array([0, 0, 3], np.int64), np.array([3, 0, 3], np.int32), np.array([1.0, 10.0, 100.0]))
    blk = O.multiply_rows(A, B)
    assert blk.col_idx.tolist() == [0, 3]
    assert blk.val.tolist() == [50.0, 505.0]
    assert O.row_products(A, B).tolist() == [6]


def test_transposed_operand_would_be_caught():
    # non-commuting rectangular shapes: A (2x3), B (3x2); result must be 2x2 and equal to dense A@B
    A_vals = np.array([[1., 2., 0.], [0., 0., 3.]]); B_vals = np.array([[4., 0.], [0., 5.], [6., 7.]])
    check_against_brute(A_vals, A_vals != 0, B_vals, B_vals != 0)


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("g", [3, 8, 33])
def test_laplacian_closed_forms_small(g):
    A = W.laplacian_2d(g)
    assert A.nnz == 5 * g * g - 4 * g
    prod = O.row_products(A, A)
    assert prod.sum() == 25 * (g - 2) ** 2 + 64 * (g - 2) + 36
    nnz = O.count_rows(A, A)
    assert nnz.sum() == g * g + 4 * g * (g - 1) + 4 * g * (g - 2) + 4 * (g - 1) ** 2


def test_laplacian_full_size_counts_and_stencil():
    g = 1024
    A = W.laplacian_2d(g)
    assert A.nnz == 5238784
    prod = O.row_products(A, A)
    assert int(prod.sum()) == 26177544 and int(prod.max()) == 25
    # squared 5-point stencil in the interior: 20 centre, -8 x4 at distance 1, 2 x4 on the
    # diagonals, 1 x4 two steps away; all integer arithmetic, hence exact
    i = 500 * g + 500
    blk = O.multiply_rows(A, A, i, i + 1)
    want = {i: 20.0, i - 1: -8.0, i + 1: -8.0, i - g: -8.0, i + g: -8.0,
            i - g - 1: 2.0, i - g + 1: 2.0, i + g - 1: 2.0, i + g + 1: 2.0,
            i - 2: 1.0, i + 2: 1.0, i - 2 * g: 1.0, i + 2 * g: 1.0}
    assert dict(zip(blk.col_idx.tolist(), blk.val.tolist())) == want
    assert blk.col_idx.tolist() == sorted(want)
    nnz = O.count_rows(A, A)
    assert int(nnz.sum()) == 13611012 and int(nnz.max()) == 13


def test_erdos_renyi_products_closed_form():
    A, B, _ = W.make("er")
    prod = O.row_products(A, B)
    assert np.all(prod == 64) and prod.sum() == 262144
    nnz = O.count_rows(A, B)
    assert nnz.max() <= 64 and nnz.min() >= 8


# ------------------------------------------------------------------ invariants
@pytest.mark.parametrize("name", ["er", "laplacian", "rmat", "rect", "clustered"])
def test_invariants_and_scipy_cross_check(name):
    A, B, _ = W.make(name, small=True)
    prod = O.row_products(A, B)
    blk = O.multiply_rows(A, B)
    nnz = np.diff(blk.row_ptr)
    n = B.cols
    assert np.all(nnz <= np.minimum(prod, n))
    blen = np.diff(B.row_ptr)
    lower = np.array([blen[A.col_idx[A.row_ptr[i]:A.row_ptr[i + 1]]].max(initial=0) for i in range(A.rows)])
    assert np.all(nnz >= lower)
    # strictly ascending columns inside every row
    d = np.diff(blk.col_idx.astype(np.int64))
    row_starts = blk.row_ptr[1:-1]
    interior = np.ones(d.shape, bool)
    interior[row_starts[(row_starts > 0) & (row_starts < blk.col_idx.size)] - 1] = False
    assert np.all(d[interior] > 0)
    # sum of products by the other counting order: sum_k colcount_A(k) * nnz(B_k)
    assert prod.sum() == int(np.dot(np.bincount(A.col_idx, minlength=A.cols).astype(np.int64), blen))
    # independent library: SciPy's sparse product (pattern via all-ones values so nothing cancels)
    SA = sp.csr_matrix((A.val.astype(np.float64), A.col_idx, A.row_ptr), shape=(A.rows, A.cols))
    SB = sp.csr_matrix((B.val.astype(np.float64), B.col_idx, B.row_ptr), shape=(B.rows, B.cols))
    PA = sp.csr_matrix((np.ones(A.nnz), A.col_idx, A.row_ptr), shape=SA.shape)
    PB = sp.csr_matrix((np.ones(B.nnz), B.col_idx, B.row_ptr), shape=SB.shape)
    PC = (PA @ PB).tocsr(); PC.sort_indices()
    assert np.array_equal(PC.indptr, blk.row_ptr) and np.array_equal(PC.indices, blk.col_idx)
    SC = (SA @ SB).tocsr(); SC.sort_indices()
    if SC.nnz == PC.nnz:   # SciPy keeps cancelled entries in @; guard anyway
        np.testing.assert_allclose(SC.data, blk.val, rtol=0, atol=1e-12 * max(1.0, blk.absval.max()))
    SabsC = (abs(SA) @ abs(SB)).tocsr(); SabsC.sort_indices()
    np.testing.assert_allclose(SabsC.data, blk.absval, rtol=1e-12)
    # C x = A (B x)
    x = np.random.default_rng(7).uniform(-1, 1, n)
    Cx = np.add.reduceat(np.append(blk.val * x[blk.col_idx], 0.0), np.minimum(blk.row_ptr[:-1], blk.val.size))
    Cx[nnz == 0] = 0.0
    np.testing.assert_allclose(Cx, SA @ (SB @ x), rtol=0, atol=1e-11 * max(1.0, blk.absval.max()) * max(1, nnz.max()))


def test_row_range_equals_full():
    A, B, _ = W.make("rmat", small=True)
    full = O.multiply_rows(A, B)
    r0, r1 = 100, 1000
    part = O.multiply_rows(A, B, r0, r1)
    s, e = full.row_ptr[r0], full.row_ptr[r1]
    assert np.array_equal(part.row_ptr, full.row_ptr[r0:r1 + 1] - s)
    assert np.array_equal(part.col_idx, full.col_idx[s:e])
    assert np.array_equal(part.val, full.val[s:e])          # same thread-independent arithmetic order per row
    empty = O.multiply_rows(A, B, 5, 5)
    assert empty.row_ptr.tolist() == [0] and empty.col_idx.size == 0


def test_rect_product_is_symmetric_with_positive_diagonal():
    A, B, _ = W.make("rect", small=True)
    blk = O.multiply_rows(A, B)
    C = sp.csr_matrix((blk.val, blk.col_idx, blk.row_ptr), shape=(A.rows, A.rows))
    D = (C - C.T).tocsr()
    assert D.nnz == 0 or np.abs(D.data).max() <= 1e-14
    assert np.array_equal((C != 0).astype(np.int8).toarray(), (C.T != 0).astype(np.int8).toarray())
    diag = C.diagonal()
    rowlen = np.diff(A.row_ptr)
    assert np.all(diag[rowlen > 0] > 0) and np.all(np.diff(blk.row_ptr)[rowlen == 0] == 0)
    sq = np.add.reduceat(np.append(A.val ** 2, 0.0), np.minimum(A.row_ptr[:-1], A.nnz)); sq[rowlen == 0] = 0
    np.testing.assert_allclose(diag, sq, rtol=1e-13)


def test_clustered_product_stays_column_stochastic():
    A, B, _ = W.make("clustered", small=True)
    assert A.val.dtype == np.float32
    blk = O.multiply_rows(A, B)
    colsum = np.bincount(blk.col_idx, weights=blk.val, minlength=B.cols)
    np.testing.assert_allclose(colsum, 1.0, rtol=0, atol=2e-5)   # inputs were rounded to float32
    assert blk.val.min() >= 0.0
    np.testing.assert_array_equal(blk.val, blk.absval)


def test_thread_count_does_not_change_results():
    A, B, _ = W.make("rect", small=True)
    O.set_threads(1); one = O.multiply_rows(A, B)
    O.set_threads(0); many = O.multiply_rows(A, B)
    assert np.array_equal(one.col_idx, many.col_idx) and np.array_equal(one.val, many.val)
