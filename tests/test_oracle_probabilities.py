"""Pins for the oracle's Algorithm 1 (Section 3) that do not go through the oracle's own formula."""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "probabilities_examples.txt")


def variance_objective(lam, p):
    lam, p = np.asarray(lam, float), np.asarray(p, float)
    nz = lam != 0
    return np.sum(lam[nz] ** 2 / p[nz])


def brute_force(lam, s):
    """eq. (opt_prob1) by enumeration: for every subset forced to p=1 the remaining atoms take the
    relaxed optimum of Lemma (opt_prob2) with the remaining budget; keep feasible candidates, return the best."""
    lam = np.abs(np.asarray(lam, float))
    n = lam.size
    best, best_p = np.inf, None
    for k in range(0, n + 1):
        if k > s:
            break
        for capped in itertools.combinations(range(n), k):
            rest = [i for i in range(n) if i not in capped]
            p = np.zeros(n)
            p[list(capped)] = 1.0
            tail = lam[rest].sum()
            budget = s - k
            if rest:
                if tail == 0 or budget <= 0:
                    continue
                p[rest] = lam[rest] * budget / tail
            elif abs(budget) > 1e-12:
                continue
            if p.max() > 1 + 1e-12 or p.min() <= 0:
                continue
            f = variance_objective(lam, p)
            if f < best - 1e-12 * max(1.0, abs(best) if np.isfinite(best) else 1.0):
                best, best_p = f, p
    return best, best_p


def kkt_by_bisection(lam, s):
    """KKT appendix: one multiplier mu with p_i = min(1, |lambda_i|/sqrt(mu)) and sum p = s."""
    a = np.abs(np.asarray(lam, float))
    lo, hi = 0.0, a.sum() / s * 4 + 1.0          # tau = sqrt(mu)
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if np.minimum(1.0, a / mid).sum() > s:
            lo = mid
        else:
            hi = mid
    return np.minimum(1.0, a / hi)


def test_hand_examples_from_golden_file():
    rows = 0
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if not line:
            continue
        s_txt, lam_txt, p_txt = [x.strip() for x in line.split("|")]
        lam = [float(x) for x in lam_txt.split()]
        want = [float(Fraction(x)) for x in p_txt.split()]
        got = oracle.probabilities(lam, float(s_txt))
        np.testing.assert_allclose(got, want, rtol=1e-14, atol=0)
        rows += 1
    assert rows >= 8


@pytest.mark.parametrize("seed", range(6))
def test_invariants_random(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 400))
    lam = rng.standard_normal(n) * np.exp(3 * rng.standard_normal(n))
    lam[rng.random(n) < 0.1] = 0.0
    nnz = int((lam != 0).sum())
    for s in (0.3, 1.0, 2.5, 7.0, n / 3 + 0.1, n - 0.5, float(n), n + 3.0):
        p, forced = oracle.probabilities(lam, s, return_forced=True)
        assert ((p >= 0) & (p <= 1)).all()
        assert (p[lam == 0] == 0).all() and (p[lam != 0] > 0).all()
        np.testing.assert_allclose(p.sum(), min(s, nnz), rtol=1e-12)
        order = np.argsort(-np.abs(lam), kind="stable")
        assert (np.diff(p[order]) <= 1e-15).all()                       # |l_i| >= |l_j|  =>  p_i >= p_j
        assert forced <= max(0, int(np.ceil(min(s, nnz))) - 1) or s >= nnz
        if s < nnz:
            assert forced <= int(np.ceil(s)) - 1
            assert (p == 1).sum() >= forced


def test_balanced_closed_form():
    # Lemma (opt_prob2) / Lemma (suff_balanced): s <= |l|_1/|l|_inf  =>  p_i = |l_i| s / |l|_1
    rng = np.random.default_rng(1)
    for _ in range(20):
        lam = rng.standard_normal(50)
        s_max = np.abs(lam).sum() / np.abs(lam).max()
        for s in (0.1, 1.0, 0.5 * s_max, s_max):
            p, forced = oracle.probabilities(lam, s, return_forced=True)
            np.testing.assert_allclose(p, np.abs(lam) * s / np.abs(lam).sum(), rtol=1e-13)
            if s < s_max:                    # at s = s_max both branches give p_max = 1; rounding picks one
                assert forced == 0
        # just above the balance limit the largest atom is forced to 1 (Theorem (all), part 2)
        p = oracle.probabilities(lam, s_max * 1.01)
        assert p[np.argmax(np.abs(lam))] == 1.0


@pytest.mark.parametrize("q", [1.0, 1.5, 2.0, 3.0, np.inf])
def test_lq_quantisation_presets(q):
    # Section 4: s = |g|_1/|g|_q  =>  p_i = |g_i|/|g|_q  (q=2: 1-bit QSGD, q=inf: TernGrad),
    # and the second moment is |g|_1 |g|_q (Theorem (lqgrad))
    rng = np.random.default_rng(2)
    g = rng.standard_normal(300) * np.exp(rng.standard_normal(300))
    nq = np.abs(g).max() if np.isinf(q) else (np.abs(g) ** q).sum() ** (1 / q)
    s = np.abs(g).sum() / nq
    p = oracle.probabilities(g, s)
    np.testing.assert_allclose(p, np.abs(g) / nq, rtol=1e-12)
    np.testing.assert_allclose(variance_objective(g, p), np.abs(g).sum() * nq, rtol=1e-12)


@pytest.mark.parametrize("seed", range(8))
def test_matches_single_multiplier_kkt(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(2, 200))
    lam = rng.standard_normal(n) * np.exp(2 * rng.standard_normal(n))
    for s in (0.7, 2.0, 3.0, 4.0, n / 4 + 0.3, n * 0.9):
        if s >= n:
            continue
        np.testing.assert_allclose(oracle.probabilities(lam, s), kkt_by_bisection(lam, s), rtol=1e-9, atol=1e-12)


def test_brute_force_small_n():
    rng = np.random.default_rng(3)
    checked_unbalanced = 0
    for trial in range(150):
        n = int(rng.integers(1, 8))
        lam = rng.standard_normal(n) * np.exp(2 * rng.standard_normal(n))
        if trial % 7 == 0 and n > 2:
            lam[1] = lam[0]                                    # ties
        s = float(rng.uniform(0.2, n))
        p, forced = oracle.probabilities(lam, s, return_forced=True)
        f_best, p_best = brute_force(lam, s)
        assert p_best is not None
        np.testing.assert_allclose(variance_objective(lam, p), f_best, rtol=1e-10)
        np.testing.assert_allclose(p, p_best, rtol=1e-9, atol=1e-12)
        checked_unbalanced += forced > 0
        # random feasible points never beat it
        for _ in range(20):
            q = rng.random(n) + 1e-3
            q *= s / q.sum()
            if q.max() <= 1:
                assert variance_objective(lam, q) >= variance_objective(lam, p) * (1 - 1e-12)
    assert checked_unbalanced > 20


def test_equivariance_scaling_and_degenerate_cases():
    rng = np.random.default_rng(4)
    lam = rng.standard_normal(64) * np.exp(2 * rng.standard_normal(64))
    p = oracle.probabilities(lam, 5.0)
    perm = rng.permutation(64)
    np.testing.assert_allclose(oracle.probabilities(lam[perm], 5.0), p[perm], rtol=1e-14)
    np.testing.assert_allclose(oracle.probabilities(-3.7 * lam, 5.0), p, rtol=1e-13)
    assert (oracle.probabilities(lam, 64.0) == 1).all()                 # s = n: no sparsification
    assert (oracle.probabilities(lam, 100.0) == 1).all()
    assert (oracle.probabilities(np.zeros(5), 2.0) == 0).all()          # all-zero gradient
    assert oracle.probabilities([], 1.0).size == 0
    np.testing.assert_allclose(oracle.probabilities([7.0], 0.25), [0.25])
    # the predicate of Algorithm 1 is monotone along the sorted order: once true, true for all later i
    for _ in range(200):
        n = int(rng.integers(2, 40))
        a = np.sort(np.abs(rng.standard_normal(n) * np.exp(2 * rng.standard_normal(n))))[::-1]
        s = float(rng.uniform(0.2, n))
        tail = np.cumsum(a[::-1])[::-1]
        pred = [a[i] * (s - i) <= tail[i] for i in range(n) if s - i > 0]
        first = pred.index(True)
        assert all(pred[first:])


def test_wide_dynamic_range_closed_form():
    # three atoms of 1e30 are forced to p = 1 (Algorithm 1); the remaining budget 2 is spread over the others in
    # proportion to their size (eq. (p_i) of the KKT appendix): tail = 3*2 + 3*1 + 2e-30, so p(2) = 4/9, p(1) = 2/9.
    # A tail sum formed by subtracting the large values from the total would lose the small ones entirely.
    lam = np.array([1e30] * 3 + [2.0] * 3 + [1.0] * 3 + [1e-30] * 2)
    want = np.array([1.0] * 3 + [4 / 9] * 3 + [2 / 9] * 3 + [2e-30 / 9] * 2)
    np.testing.assert_allclose(oracle.probabilities(lam, 5.0), want, rtol=1e-14)
    perm = np.random.default_rng(0).permutation(lam.size)
    np.testing.assert_allclose(oracle.probabilities(lam[perm], 5.0), want[perm], rtol=1e-14)
