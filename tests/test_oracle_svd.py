"""Pins for the oracle's SVD (Section 5, Notation: X = sum sigma_i u_i v_i^T)."""
import numpy as np
import pytest

import oracle
from paper_1806_04090_amd import inputs


def householder_orthonormal(rng, dim, k):
    q, _ = np.linalg.qr(rng.standard_normal((dim, k)))      # LAPACK Householder QR
    return q


def check_factorisation(G, sigma, U, V, tol=1e-12):
    m, n = G.shape
    r = min(m, n)
    assert sigma.shape == (r,) and U.shape == (m, r) and V.shape == (n, r)
    assert (np.diff(sigma) <= 0).all() and (sigma >= 0).all()
    scale = max(sigma[0], 1e-300)
    assert np.abs(U.T @ U - np.eye(r)).max() < tol
    assert np.abs(V.T @ V - np.eye(r)).max() < tol
    assert np.linalg.norm(G - (U * sigma) @ V.T) <= tol * max(np.linalg.norm(G), 1e-300) * 10
    # per-atom residuals: G v_i = sigma_i u_i and G^T u_i = sigma_i v_i
    assert np.abs(G @ V - U * sigma).max() < tol * scale * 10
    assert np.abs(G.T @ U - V * sigma).max() < tol * scale * 10


@pytest.mark.parametrize("m,n", [(1, 1), (1, 7), (7, 1), (5, 5), (12, 40), (40, 12), (64, 27), (33, 70)])
def test_prescribed_singular_values(m, n):
    rng = np.random.default_rng(m * 1000 + n)
    r = min(m, n)
    want = np.sort(np.exp(rng.uniform(-6, 2, size=r)))[::-1]
    G = (householder_orthonormal(rng, m, r) * want) @ householder_orthonormal(rng, n, r).T
    sigma, U, V = oracle.svd(G)
    np.testing.assert_allclose(sigma, want, rtol=1e-11)
    check_factorisation(G, sigma, U, V)


def test_two_by_two_closed_form():
    a, b, c, d = 3.0, -1.0, 2.0, 0.5
    G = np.array([[a, b], [c, d]])
    fro2, det = a * a + b * b + c * c + d * d, abs(a * d - b * c)
    s1 = np.sqrt((fro2 + np.sqrt(fro2 * fro2 - 4 * det * det)) / 2)
    sigma, U, V = oracle.svd(G)
    np.testing.assert_allclose(sigma, [s1, det / s1], rtol=1e-14)
    check_factorisation(G, sigma, U, V)


def test_extremal_matrices_of_the_norm_appendix():
    # Appendix (equivalence of norms): e1 e1^T has sigma = (1, 0, ...); all-ones n x m has the single value sqrt(nm)
    for m, n in [(4, 6), (6, 4), (9, 9)]:
        E = np.zeros((m, n)); E[0, 0] = 1.0
        sigma, U, V = oracle.svd(E)
        np.testing.assert_allclose(sigma, [1.0] + [0.0] * (min(m, n) - 1), atol=1e-15)
        check_factorisation(E, sigma, U, V)
        sigma, U, V = oracle.svd(np.ones((m, n)))
        np.testing.assert_allclose(sigma, [np.sqrt(m * n)] + [0.0] * (min(m, n) - 1), atol=1e-13)
        check_factorisation(np.ones((m, n)), sigma, U, V)
    sigma, _, _ = oracle.svd(np.zeros((3, 5)))
    assert (sigma == 0).all()


def test_diagonal_and_permutation_matrices():
    rng = np.random.default_rng(5)
    d = np.array([0.5, -3.0, 2.0, 1e-3, 7.0])
    G = np.zeros((5, 8)); G[np.arange(5), [3, 0, 7, 1, 4]] = d        # scaled partial permutation
    sigma, U, V = oracle.svd(G)
    np.testing.assert_allclose(sigma, np.sort(np.abs(d))[::-1], rtol=1e-14)
    check_factorisation(G, sigma, U, V)
    P = np.eye(6)[rng.permutation(6)]
    sigma, U, V = oracle.svd(P)
    np.testing.assert_allclose(sigma, np.ones(6), rtol=1e-14)


@pytest.mark.parametrize("case", ["gauss_wide", "gauss_tall", "cfg1", "resnet_small_layers"])
def test_against_lapack(case):
    rng = np.random.default_rng(6)
    if case == "gauss_wide":
        mats = [rng.standard_normal((20, 90))]
    elif case == "gauss_tall":
        mats = [rng.standard_normal((90, 20))]
    elif case == "cfg1":
        mats = [inputs.single_conv_layer(0).astype(np.float64)]
    else:
        mats = [g.astype(np.float64) for g in inputs.resnet18_layer_set(0, shapes=[(64, 27), (128, 64), (10, 512)])]
    for G in mats:
        sigma, U, V = oracle.svd(G)
        np.testing.assert_allclose(sigma, np.linalg.svd(G, compute_uv=False), rtol=1e-11)
        check_factorisation(G, sigma, U, V)


def test_norm_lemma():
    # Lemma (compare_norms): |X|_{1,1}/sqrt(nm) <= |X|_* <= |X|_{1,1}
    rng = np.random.default_rng(7)
    for _ in range(20):
        m, n = int(rng.integers(1, 12)), int(rng.integers(1, 12))
        X = rng.standard_normal((m, n)) * np.exp(rng.standard_normal((m, n)))
        nuc = oracle.svd(X)[0].sum()
        l11 = np.abs(X).sum()
        assert l11 / np.sqrt(m * n) <= nuc * (1 + 1e-12)
        assert nuc <= l11 * (1 + 1e-12)


def test_planted_signal_is_recovered():
    # cfg-like input: planted unit vectors come back (up to sign) where the gap to the noise is large
    rng = np.random.default_rng(8)
    m, n = 24, 60
    u = householder_orthonormal(rng, m, 2)
    v = householder_orthonormal(rng, n, 2)
    G = (u * [1.0, 0.5]) @ v.T + 1e-6 * rng.standard_normal((m, n))
    sigma, U, V = oracle.svd(G)
    np.testing.assert_allclose(sigma[:2], [1.0, 0.5], rtol=1e-4)
    for k in range(2):
        np.testing.assert_allclose(np.outer(U[:, k], V[:, k]), np.outer(u[:, k], v[:, k]), atol=1e-4)
