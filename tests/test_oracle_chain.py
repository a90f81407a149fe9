"""Pins for the oracle's sampling, rescaling and decoding (eq. (vhat), Lemma (basic), Theorem (all))."""
import numpy as np
import pytest

import oracle
from paper_1806_04090_amd import inputs


def test_decode_svd_is_the_rank_one_sum():
    rng = np.random.default_rng(0)
    m, n, k = 5, 7, 3
    msg = {"w": rng.standard_normal(k), "U": rng.standard_normal((m, k)), "V": rng.standard_normal((n, k))}
    want = np.einsum("k,ik,jk->ij", msg["w"], msg["U"], msg["V"])
    np.testing.assert_allclose(oracle.decode_svd([msg], m, n), want, rtol=1e-13, atol=1e-15)
    # several messages and a scale: mean of the single decodes (parameter-server average, Section 2)
    msg2 = {"w": rng.standard_normal(2), "U": rng.standard_normal((m, 2)), "V": rng.standard_normal((n, 2))}
    empty = {"w": np.zeros(0), "U": np.zeros((m, 0)), "V": np.zeros((n, 0))}
    mean = (oracle.decode_svd([msg], m, n) + oracle.decode_svd([msg2], m, n)) / 3
    np.testing.assert_allclose(oracle.decode_svd([msg, msg2, empty], m, n, scale=1 / 3), mean, rtol=1e-13, atol=1e-15)


def test_decode_entrywise_is_a_scatter():
    got = oracle.decode_entrywise([{"idx": [1, 4], "val": [2.0, -3.0]}, {"idx": [4], "val": [10.0]}], 6, scale=0.5)
    np.testing.assert_array_equal(got, [0, 1.0, 0, 0, 3.5, 0])


def test_full_budget_returns_the_gradient_exactly():
    # KKT appendix, consequence 1: s >= n means p = 1 everywhere, nothing is dropped
    G = inputs.low_rank_plus_noise(np.random.default_rng(1), 12, 30, [1.0, 0.3], 1e-2)
    enc = oracle.encode_svd(G, s=12, seed=3, stream=1)
    assert enc["mask"].all() and np.allclose(enc["w"], enc["sigma"])
    np.testing.assert_allclose(oracle.decode_svd([enc], 12, 30), G.astype(np.float64), atol=1e-13)
    g = G.ravel()
    enc = oracle.encode_entrywise(g, s=g.size + 5, seed=3, stream=1)
    assert np.array_equal(enc["idx"], np.arange(g.size))
    np.testing.assert_array_equal(oracle.decode_entrywise([enc], g.size), g.astype(np.float64))


def test_kept_uncapped_weights_are_one_constant():
    # eq. (p_i) of the KKT appendix: lambda_i/p_i = sum_{j>n_s}|lambda_j| / (s - n_s) for every uncapped atom
    lam = np.array([50.0, -20.0, 3.0, -2.0, 1.5, 1.0, -0.5, 0.25] * 40)
    s = 100.0
    p, forced = oracle.probabilities(lam, s, return_forced=True)
    assert forced == 80
    mask = oracle.bernoulli_mask(p.astype(np.float32), 7, 0)
    idx, w = oracle.pack_weights(lam, p, mask)
    assert np.array_equal(idx, np.flatnonzero(mask))
    capped = np.abs(lam[idx]) >= 20
    np.testing.assert_array_equal(w[capped], lam[idx][capped])
    const = np.abs(lam)[np.abs(lam) < 20].sum() / (s - forced)
    np.testing.assert_allclose(w[~capped], np.sign(lam[idx][~capped]) * const, rtol=1e-13)


def _z(sample_mean, true_mean, sample_var, trials):
    return (sample_mean - true_mean) / np.sqrt(np.maximum(sample_var, 1e-300) / trials)


def test_spectral_estimator_is_unbiased_with_the_stated_second_moment():
    # Lemma (basic): E[g_hat] = g and E|g_hat|^2 = sum sigma_i^2/p_i (orthonormal atoms: no cross terms);
    # also E[k] = s and Var[k] = sum p(1-p)
    G = inputs.low_rank_plus_noise(np.random.default_rng(2), 6, 9, [1.0, 0.4], 5e-2).astype(np.float64)
    s = 2.0
    sigma, U, V = oracle.svd(G)
    p = oracle.probabilities(sigma, s)
    trials = 20_000
    acc = np.zeros_like(G); acc2 = np.zeros_like(G); norms = np.zeros(trials); counts = np.zeros(trials)
    for t in range(trials):
        enc = oracle.encode_svd(G, s, seed=99, stream=t, sigma_UV=(sigma, U, V))
        gh = oracle.decode_svd([enc], 6, 9)
        acc += gh; acc2 += gh * gh; norms[t] = (gh * gh).sum(); counts[t] = enc["idx"].size
    mean = acc / trials
    var = acc2 / trials - mean ** 2
    z = _z(mean, G, var, trials)
    assert np.abs(z).max() < 4.5
    want2 = (sigma ** 2 / p).sum()
    assert abs(_z(norms.mean(), want2, norms.var(), trials)) < 4.5
    assert abs(_z(counts.mean(), s, counts.var(), trials)) < 4.5
    np.testing.assert_allclose(counts.var(), (p * (1 - p)).sum(), rtol=0.05)


def test_entrywise_estimator_is_unbiased_and_balanced_second_moment():
    # Theorem (all), part 1: balanced  =>  E|g_hat|^2 = |lambda|_1^2 / s  (standard basis: no cross terms)
    rng = np.random.default_rng(3)
    g = rng.standard_normal(40)
    s = 4.0
    assert s <= np.abs(g).sum() / np.abs(g).max()
    trials = 20_000
    acc = np.zeros(40); acc2 = np.zeros(40); norms = np.zeros(trials)
    for t in range(trials):
        enc = oracle.encode_entrywise(g, s, seed=5, stream=t)
        gh = oracle.decode_entrywise([enc], 40)
        acc += gh; acc2 += gh * gh; norms[t] = (gh * gh).sum()
    mean = acc / trials
    z = _z(mean, g, acc2 / trials - mean ** 2, trials)
    assert np.abs(z).max() < 4.5
    assert abs(_z(norms.mean(), np.abs(g).sum() ** 2 / s, norms.var(), trials)) < 4.5


def test_unbalanced_entrywise_estimator_is_unbiased():
    g = np.array([10.0, -6.0, 0.5, 0.25, -0.25, 0.125, 0.0, 1.0])
    s = 3.0
    p = oracle.probabilities(g, s)
    assert (p[:2] == 1).all() and p[6] == 0
    trials = 20_000
    acc = np.zeros(8); acc2 = np.zeros(8)
    for t in range(trials):
        gh = oracle.decode_entrywise([oracle.encode_entrywise(g, s, seed=1, stream=t)], 8)
        acc += gh; acc2 += gh * gh
    mean = acc / trials
    var = acc2 / trials - mean ** 2
    assert (mean[[0, 1, 6]] == g[[0, 1, 6]]).all()                 # capped and zero atoms are deterministic
    free = [2, 3, 4, 5, 7]
    assert np.abs(_z(mean[free], g[free], var[free], trials)).max() < 4.5


def test_same_seed_same_message_and_ascending_indices():
    g = inputs.flat_heavy_tail(seed=0, n=20_000)
    a = oracle.encode_entrywise(g, 200.0, seed=0, stream=0)
    b = oracle.encode_entrywise(g, 200.0, seed=0, stream=0)
    assert np.array_equal(a["idx"], b["idx"]) and np.array_equal(a["val"], b["val"])
    assert (np.diff(a["idx"]) > 0).all()
    c = oracle.encode_entrywise(g, 200.0, seed=0, stream=1)
    assert not np.array_equal(a["idx"], c["idx"])
    assert abs(a["idx"].size - 200) < 6 * np.sqrt(200)


def test_folded_message_decodes_to_the_same_matrix_and_costs_s_times_n_plus_m():
    # Table "matrix_sparse": the SVD sparsification communicates s(n + m) reals in expectation
    G = inputs.single_conv_layer(0).astype(np.float64)
    msg = oracle.encode_svd(G, 2.0, 0, 0)
    folded = oracle.fold_svd_message(msg)
    assert folded["w"] is None
    np.testing.assert_allclose(oracle.decode_svd([folded], *G.shape), oracle.decode_svd([msg], *G.shape), atol=1e-14)
    np.testing.assert_allclose(np.linalg.norm(folded["U"], axis=0), msg["w"], rtol=1e-12)
    reals = folded["U"].size + folded["V"].size
    assert reals == msg["idx"].size * (G.shape[0] + G.shape[1])
    assert abs(msg["p"].sum() - 2.0) < 1e-12                      # so E[reals] = s (n + m)


def test_ps_update_with_full_budget_is_plain_minibatch_sgd():
    # s >= rank: every atom is kept with p = 1 (KKT appendix), each message decodes to its gradient, and the
    # step of Section 2 becomes w - gamma * mean of the workers' gradients
    rng = np.random.default_rng(3)
    shapes = [(12, 20), (30, 7)]
    P, gamma = 4, 0.1
    params = [rng.standard_normal(sh) for sh in shapes]
    grads = [[rng.standard_normal(sh) for _ in range(P)] for sh in shapes]
    msgs = [[oracle.encode_svd(g, float(min(sh)), 5, 100 * l + k) for k, g in enumerate(gl)]
            for l, (sh, gl) in enumerate(zip(shapes, grads))]
    new = oracle.ps_update(params, msgs, gamma)
    for w, gl, got in zip(params, grads, new):
        np.testing.assert_allclose(got, w - gamma * np.mean(gl, axis=0), atol=1e-12)
    # folded messages give the same step
    folded = [[oracle.fold_svd_message(m) for m in ml] for ml in msgs]
    for a, b in zip(oracle.ps_update(params, folded, gamma), new):
        np.testing.assert_allclose(a, b, atol=1e-13)


def test_ps_update_is_unbiased_in_expectation():
    # E[g_hat] = g (unbiasedness, Section 3): averaged over many seeds the sparsified step approaches the dense one
    rng = np.random.default_rng(8)
    G = inputs.low_rank_plus_noise(rng, 16, 24, [1.0, 0.5, 0.25], 0.05).astype(np.float64)
    w0 = rng.standard_normal(G.shape)
    svd_parts = oracle.svd(G)
    trials = 4000
    acc = np.zeros_like(G)
    for t in range(trials):
        msg = oracle.encode_svd(G, 2.0, t, 0, sigma_UV=svd_parts)
        acc += oracle.ps_update([w0], [[msg]], 0.5)[0]
    mean_step = acc / trials
    # standard error of the mean of the step: gamma * sqrt(E|g_hat - g|^2 / trials), bounded by the variance term
    sig, p = svd_parts[0], oracle.probabilities(svd_parts[0], 2.0)
    var = np.sum(sig ** 2 * (1.0 / np.maximum(p, 1e-300) - 1.0) * (p > 0))
    assert np.linalg.norm(mean_step - (w0 - 0.5 * G)) <= 0.5 * 4.0 * np.sqrt(var / trials)
