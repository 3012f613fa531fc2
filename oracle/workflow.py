"""Analysis-step reference: statistics, sampling and workflow choice.
TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

Section 3.2 defines the statistics (input expansion ratio ER = products /
nnz(A); output compression ratio CR = products / nnz(C); sampled CR from
merged sketches of a subset of A's rows), Section 4.3 fixes the parameters
(register count, sampling ratio and limits, thresholds) and Table 1 the
selection rule.
"""
from __future__ import annotations

import math

import numpy as np

UPPER_BOUND, HLL, SYMBOLIC = 1, 2, 3   # workflow ids (0 is "auto" at the library boundary)


def hll_registers(er: float) -> int:
    """Section 4.3: 32 registers when ER < 48, else 64."""
    return 32 if er < 48.0 else 64


def expansion_coef(m: int) -> float:
    """Section 5.3: estimates are multiplied by 1.5 before binning, 2.0 with 32 registers."""
    return 2.0 if m == 32 else 1.5


def sample_size(rows: int) -> int:
    """Section 4.3: 3 % of A's rows, at least 600 and at most 10 000 (never more than there are)."""
    return min(rows, max(600, min(10000, math.ceil(0.03 * rows))))


def _fmix32(x: int) -> int:
    x &= 0xFFFFFFFF
    x ^= x >> 16
    x = (x * 0x85EBCA6B) & 0xFFFFFFFF
    x ^= x >> 13
    x = (x * 0xC2B2AE35) & 0xFFFFFFFF
    x ^= x >> 16
    return x


def sample_rows(rows: int, seed: int) -> np.ndarray:
    """Stratified pseudo-random sample: the t-th of n_s equal strata of the row
    range contributes one row, picked by a counter-based hash of (seed, t)."""
    ns = sample_size(rows)
    out = np.empty(ns, dtype=np.int64)
    for t in range(ns):
        lo = t * rows // ns
        hi = (t + 1) * rows // ns
        out[t] = lo + _fmix32((seed + 0x9E3779B9 * (t + 1)) & 0xFFFFFFFF) % (hi - lo)
    return out


def sampled_cr(prod_s: np.ndarray, est_s: np.ndarray) -> float:
    """Ratio of sums over the sampled rows (the global definition of CR applied
    to the sample); rows with no output are skipped; 1.0 when nothing is left."""
    keep = est_s > 0
    den = float(np.sum(est_s[keep]))
    return float(np.sum(prod_s[keep])) / den if den > 0 else 1.0


def conservative_cr(prod_s: np.ndarray, est_s: np.ndarray, sigmas: float = 1.0) -> tuple[float, float, float]:
    """Section 4.1 (assisted symbolic step): mean and standard deviation of the compression ratio over the
    sampled rows, and a conservative ratio for the whole matrix.  The paper does not print how the two are
    combined; the reading taken: per-row ratios products / estimate (rows with no output skipped), their
    arithmetic mean mu and population standard deviation sigma, conservative CR = max(1, mu - sigmas*sigma).
    Returns (mu, sigma, conservative)."""
    keep = est_s > 0
    if not np.any(keep):
        return 0.0, 0.0, 1.0
    r = prod_s[keep].astype(np.float64) / est_s[keep].astype(np.float64)
    mu = float(np.mean(r))
    sigma = float(np.sqrt(np.mean((r - mu) ** 2)))
    return mu, sigma, max(1.0, mu - sigmas * sigma)


def select_workflow(avg_products: float, er: float, cr: float) -> int:
    """Table 1."""
    if avg_products < 64.0:
        return UPPER_BOUND
    if er >= 8.0 and cr >= 8.0:
        return HLL
    return SYMBOLIC


def select_workflow_tuned(avg_products: float, er: float, cr: float, products: float, heavy_products: float,
                          cr_light: float = 3.0, cr_heavy: float = 4.5, min_products: float = 4194304.0,
                          cr_bound: float = 1.5) -> int:
    """Table 1 with the CR threshold re-derived for one GPU (not in the paper; Section 4.3 says the 8 was chosen
    empirically to amortize compaction): the threshold slides linearly from cr_light to cr_heavy with the
    share of the products held by rows that outgrow the on-chip hash tables; small problems take the two-pass
    workflow whatever the ratios (no sample is taken for them).
    Where the estimation workflow would be chosen at a CR below cr_bound, the upper-bound workflow is: the
    product bound is then as tight a reservation as an estimate with its expansion factor."""
    if avg_products < 64.0:
        return UPPER_BOUND
    if products < min_products:
        return SYMBOLIC
    share = heavy_products / products if products > 0 else 0.0
    thr = cr_light + (cr_heavy - cr_light) * share
    if er >= 8.0 and cr >= thr:
        return UPPER_BOUND if cr < cr_bound else HLL
    return SYMBOLIC


def rel_var_inv_cr(n_sampled: int, m: int, cv: float) -> float:
    """Section 4.3: relative variance of 1/CR from n_sampled rows."""
    eps = 1.04 / math.sqrt(m)
    return (eps * eps + cv * cv * (1.0 + eps * eps)) / n_sampled


def chebyshev_rel_error(n_sampled: int, m: int, cv: float, confidence: float = 0.95) -> float:
    """Chebyshev bound on the relative error at the given confidence."""
    k = 1.0 / math.sqrt(1.0 - confidence)
    return k * math.sqrt(rel_var_inv_cr(n_sampled, m, cv))
