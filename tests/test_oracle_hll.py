"""Pins for the HyperLogLog / analysis oracle: statistical error against the
paper's figures, exact special cases, merge algebra, Table 1 and the worked
sampling-error example.  CPU only."""
import math

import numpy as np
import pytest

from oracle import hll, workflow as wf
from oracle import spgemm as O
from paper_2604_19004_amd import workloads as W


def _golden(path):
    rows = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def test_hash_is_a_bijection_with_avalanche():
    x = np.arange(1 << 20, dtype=np.int64)
    h = hash_ = hll.hash32(x)
    assert hash_.dtype == np.uint32 and np.unique(h).size == x.size
    # flipping one input bit flips about half of the output bits
    flips = np.unpackbits((hll.hash32(x ^ 1) ^ h).view(np.uint8)).mean() * 32
    assert 14.0 < flips < 18.0
    # low bits (register index) are uniform over consecutive ids
    cnt = np.bincount((h & np.uint32(63)).astype(np.int64), minlength=64)
    assert cnt.min() > 0.95 * x.size / 64 and cnt.max() < 1.05 * x.size / 64


def test_rank_distribution_is_geometric():
    # P(rank = r) = 2^-r for a uniform hash: this pins the "+1" and the bit order of the rank
    _, rank = hll.index_and_rank(np.arange(1 << 20), 64)
    n = rank.size
    for r in (1, 2, 3, 4, 5):
        assert abs(np.mean(rank == r) - 2.0 ** -r) < 4 * math.sqrt(2.0 ** -r / n)
    assert rank.min() >= 1 and rank.max() <= 32 - 6 + 1


def test_rank_and_index_by_hand():
    m = 64
    for c in (0, 1, 12345, 2 ** 31 - 1):
        h = int(hll.hash32(np.array([c]))[0])
        bits = format(h, "032b")
        idx = int(bits[-6:], 2)                        # low 6 bits
        rest = bits[:-6]                               # remaining 26 bits, most significant first
        rank = (rest.index("1") + 1) if "1" in rest else 27
        i, r = hll.index_and_rank(np.array([c]), m)
        assert (int(i[0]), int(r[0])) == (idx, rank)


def test_estimate_special_cases():
    for m in (32, 64, 128):
        assert hll.estimate(np.zeros(m, np.uint8)) == 0.0                       # empty set
        one = np.zeros(m, np.uint8); one[3] = 5
        assert hll.estimate(one) == pytest.approx(m * math.log(m / (m - 1)))     # linear counting, ~1
        assert 1.0 < hll.estimate(one) < 1.02
        full = np.full(m, 10, np.uint8)                                           # no empty register
        assert hll.estimate(full) == pytest.approx(hll.alpha(m) * m * 2 ** 10)
    # small sets are counted almost exactly by linear counting
    for n in (1, 2, 5, 10):
        e = hll.estimate(hll.sketch(np.arange(100, 100 + n), 64))
        assert abs(e - n) <= 0.6 + 0.1 * n


@pytest.mark.parametrize("m", [32, 64, 128])
def test_relative_error_matches_theory_and_paper(m, golden_dir):
    rng = np.random.default_rng(100 + m)
    paper = {int(a): float(b) for a, b in _golden(golden_dir + "/hll_mean_error.txt")}
    trials, errs = 1200, []
    for n in (2000, 20000):
        for _ in range(trials // 2):
            ids = np.unique(rng.integers(0, 1 << 31, size=n))
            errs.append(hll.estimate(hll.sketch(ids, m)) / ids.size - 1.0)
    errs = np.array(errs)
    sigma = 1.04 / math.sqrt(m)                                 # Section 2.4
    assert abs(errs.mean()) < 4 * sigma / math.sqrt(trials)    # unbiased
    assert 0.85 * sigma < errs.std() < 1.15 * sigma
    # Section 5.3 reports 0.13 / 0.10 / 0.07 mean per-row error; mean |N(0, sigma)| = 0.8 sigma
    assert abs(np.abs(errs).mean() - paper[m]) < 0.03


def test_merge_algebra_and_duplicates():
    rng = np.random.default_rng(5)
    X = rng.integers(0, 10 ** 6, 500); Y = rng.integers(0, 10 ** 6, 700)
    for m in (32, 64):
        sx, sy = hll.sketch(X, m), hll.sketch(Y, m)
        assert np.array_equal(hll.sketch(np.concatenate([X, Y]), m), np.maximum(sx, sy))
        assert np.array_equal(hll.sketch(np.concatenate([X, X, X]), m), sx)


@pytest.mark.parametrize("name", ["er", "rmat", "rect"])
def test_construct_and_merge_equals_direct_sketch(name):
    A, B, _ = W.make(name, small=True)
    m = 64
    S = hll.sketch_rows(B, m)
    rows = np.arange(0, A.rows, max(1, A.rows // 200))
    merged = hll.merge_rows(A, S, rows)
    for t, i in enumerate(rows):
        ks = A.col_idx[A.row_ptr[i]:A.row_ptr[i + 1]]
        allcols = np.concatenate([B.col_idx[B.row_ptr[k]:B.row_ptr[k + 1]] for k in ks]) if ks.size else np.zeros(0, np.int32)
        assert np.array_equal(merged[t], hll.sketch(allcols, m))


def test_estimates_track_exact_row_sizes():
    A, B, _ = W.make("clustered", small=True)
    nnz = O.count_rows(A, B)
    prod = O.row_products(A, B)
    for m in (32, 64, 128):
        est = hll.estimate_rows(A, B, m)
        rel = np.abs(est - nnz) / np.maximum(nnz, 1)
        assert rel.mean() < 1.1 * 1.04 / math.sqrt(m)
        assert np.all(est <= np.minimum(prod, B.cols))
    # overflow ratio with the paper's expansion (Section 5.3): rows whose true size exceeds 80 % of coef*est
    est = hll.estimate_rows(A, B, 64)
    over = np.mean(nnz > 0.8 * 1.5 * est)
    assert over < 0.10


def test_parameters_match_paper_table(golden_dir):
    g = {k: float(v) for k, v in _golden(golden_dir + "/workflow_table.txt")}
    t_avg, t_er, t_cr = g["upper_bound_if_avg_products_below"], g["hll_if_er_at_least"], g["hll_if_cr_at_least"]
    assert wf.select_workflow(t_avg - 1e-9, 100, 100) == wf.UPPER_BOUND
    assert wf.select_workflow(t_avg, t_er, t_cr) == wf.HLL                    # all three bounds inclusive
    assert wf.select_workflow(t_avg, t_er - 1e-9, t_cr) == wf.SYMBOLIC
    assert wf.select_workflow(t_avg, t_er, t_cr - 1e-9) == wf.SYMBOLIC
    assert wf.select_workflow(1e9, 1e9, 1.0) == wf.SYMBOLIC
    assert wf.hll_registers(48 - 1e-9) == g["registers_if_er_below_48"] and wf.hll_registers(48) == g["registers_otherwise"]
    assert wf.sample_size(10 ** 5) == math.ceil(g["sampling_ratio"] * 10 ** 5)
    assert wf.sample_size(1000) == g["sampling_min_rows"] and wf.sample_size(10 ** 7) == g["sampling_max_rows"]
    assert wf.sample_size(100) == 100
    assert wf.expansion_coef(32) == 2.0 and wf.expansion_coef(64) == 1.5


def test_sampled_cr_error_worked_example(golden_dir):
    n_s = wf.sample_size(200000)
    assert n_s == 6000
    for cv, bound in _golden(golden_dir + "/sampled_cr_error.txt"):
        e = wf.chebyshev_rel_error(n_s, 64, float(cv))
        assert e < float(bound) + 0.006 and e > float(bound) - 0.01       # the text rounds to whole percent


def test_sample_rows_are_stratified_and_repeatable():
    for rows in (100, 4096, 1 << 20):
        s = wf.sample_rows(rows, seed=11)
        assert s.size == wf.sample_size(rows)
        assert np.all(np.diff(s) > 0) and s.min() >= 0 and s.max() < rows
        assert np.array_equal(s, wf.sample_rows(rows, seed=11))
    assert not np.array_equal(wf.sample_rows(4096, 1), wf.sample_rows(4096, 2))


def test_sampled_cr_close_to_true_cr():
    A, B, _ = W.make("clustered", small=True)
    prod = O.row_products(A, B); nnz = O.count_rows(A, B)
    rows = wf.sample_rows(A.rows, seed=3)
    est = hll.estimate_rows(A, B, 64, rows=rows)
    cr_s = wf.sampled_cr(prod[rows].astype(np.float64), est)
    cr = prod.sum() / nnz.sum()
    assert abs(cr_s / cr - 1) < 0.1


def test_conservative_cr_by_hand():
    # Section 4.1 as read here: ratios 2, 4, 3 -> mean 3, population std sqrt(2/3); an empty row is skipped
    prod = np.array([10, 20, 30, 0], np.float64)
    est = np.array([5, 5, 10, 0], np.float64)
    mu, sigma, cons = wf.conservative_cr(prod, est)
    assert mu == pytest.approx(3.0) and sigma == pytest.approx(math.sqrt(2.0 / 3.0))
    assert cons == pytest.approx(3.0 - math.sqrt(2.0 / 3.0))
    assert wf.conservative_cr(prod, est, sigmas=2.0)[2] == pytest.approx(3.0 - 2.0 * math.sqrt(2.0 / 3.0))
    assert wf.conservative_cr(prod, est, sigmas=10.0)[2] == 1.0                      # never below 1: nnz <= products
    assert wf.conservative_cr(np.zeros(3), np.zeros(3)) == (0.0, 0.0, 1.0)
    # identical rows: no spread, the conservative ratio is the ratio itself
    assert wf.conservative_cr(np.full(7, 12.0), np.full(7, 4.0)) == (3.0, 0.0, 3.0)

