"""Pins for the oracle's l_q quantisation (Section 4: 1-bit QSGD, TernGrad, Theorem (lqgrad)).

The closed form p_i = |g_i| / ||g||_q is checked against things it does not compute itself: Algorithm 1 run
at the budget the section derives (the two must agree because every g is s-balanced for that s), numpy's
norms, the theorem's second moment, and the estimator's mean over seeds."""
import numpy as np
import pytest

import oracle


def gradient(seed, n=5000):
    rng = np.random.default_rng(seed)
    g = rng.standard_normal(n) * np.exp(rng.standard_normal(n))
    g[rng.random(n) < 0.05] = 0.0
    return g


@pytest.mark.parametrize("q", [0.5, 1.0, 1.5, 2.0, 3.0, 8.0, float("inf")])
def test_norm_matches_numpy_and_probabilities_are_valid(q):
    g = gradient(1)
    p, norm = oracle.lq_probabilities(g, q)
    want = np.abs(g).max() if np.isinf(q) else (np.abs(g) ** q).sum() ** (1.0 / q)
    np.testing.assert_allclose(norm, want, rtol=1e-12)
    assert (p >= 0).all() and (p[g == 0] == 0).all()
    assert p.max() <= 1.0                         # |g_i| <= ||g||_inf <= ||g||_q: a valid probability (Section 4)
    np.testing.assert_allclose(p.sum(), np.abs(g).sum() / norm, rtol=1e-12)      # s = ||g||_1 / ||g||_q


@pytest.mark.parametrize("q", [1.0, 2.0, 4.0, float("inf")])
def test_agrees_with_algorithm_1_at_the_sections_budget(q):
    # every g is s-balanced for s = ||g||_1 / ||g||_q, so Algorithm 1 must return |g| / ||g||_q
    g = gradient(2, n=3000)
    p, norm = oracle.lq_probabilities(g, q)
    s = np.abs(g).sum() / norm
    p_alg1, forced = oracle.probabilities(g, s, return_forced=True)
    np.testing.assert_allclose(p_alg1, p, rtol=1e-10, atol=1e-15)


def test_qsgd_and_terngrad_special_cases():
    g = gradient(3)
    np.testing.assert_allclose(oracle.lq_probabilities(g, 2.0)[0], np.abs(g) / np.linalg.norm(g), rtol=1e-12)
    np.testing.assert_allclose(oracle.lq_probabilities(g, float("inf"))[0], np.abs(g) / np.abs(g).max(), rtol=1e-12)
    assert oracle.lq_probabilities(np.zeros(7), 2.0)[1] == 0.0 and (oracle.lq_probabilities(np.zeros(7), 2.0)[0] == 0).all()


@pytest.mark.parametrize("q", [2.0, float("inf")])
def test_second_moment_of_theorem_lqgrad_and_unbiasedness(q):
    # E ||L_q(g)||^2 = ||g||_1 ||g||_q  and  E L_q(g) = g, over independent Philox streams
    g = gradient(4, n=400)
    p, norm = oracle.lq_probabilities(g, q)
    trials = 4000
    acc = np.zeros_like(g)
    sq = 0.0
    for t in range(trials):
        m = oracle.encode_lq(g, q, seed=9, stream=t)
        out = oracle.decode_lq([m], g.size)
        acc += out
        sq += (out ** 2).sum()
    want_sq = np.abs(g).sum() * norm
    var_sq = (norm ** 4) * (p * (1 - p)).sum()                 # variance of sum_i norm^2 t_i
    assert abs(sq / trials - want_sq) < 5 * np.sqrt(var_sq / trials)
    sd = norm * np.sqrt(p * (1 - p) / trials)
    live = p * trials >= 30
    assert (np.abs(acc / trials - g)[live] <= 5.5 * sd[live] + 1e-12 * norm).all()      # (p = 1: no spread at all)
    assert np.abs((acc / trials - g).sum()) < 5 * np.sqrt((sd ** 2).sum())


def test_message_fields_and_decode():
    g = np.array([3.0, -4.0, 0.0, 1e-3, -12.0])
    m = oracle.encode_lq(g, float("inf"), seed=1, stream=0)
    assert m["norm"] == 12.0 and m["mask"][4] and not m["mask"][2]          # p = 1 is always kept, p = 0 never
    assert (m["sign"] == np.sign(g[m["idx"]])).all()
    out = oracle.decode_lq([m, m], g.size, scale=0.5)
    assert (out[m["idx"]] == m["sign"] * 12.0).all() and (np.delete(out, m["idx"]) == 0).all()
