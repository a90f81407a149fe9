"""Helpers shared by the GPU parity tests (not collected by pytest)."""
import numpy as np
import torch

import oracle
from paper_1806_04090_amd import binding

_ctx = None


def ctx():
    global _ctx
    if _ctx is None:
        _ctx = binding.Context(0)
    return _ctx


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def sigma_tolerance_ok(got, want):
    """|got - want| <= 1e-4 * max(want, 1e-3 * want_max): relative 1e-4, floored for tiny singular values."""
    want = np.asarray(want, dtype=np.float64)
    floor = 1e-3 * (want.max() if want.size else 0.0)
    return np.abs(np.asarray(got, dtype=np.float64) - want) <= 1e-4 * np.maximum(want, floor) + 1e-30


def check_svd_message_against_matrix(G, host_msg, sigma_gpu, p_gpu, tol=1e-4):
    """Properties any correct Spectral-ATOMO message has, whatever basis was picked inside sigma clusters."""
    G = np.asarray(G, dtype=np.float64)
    idx, w = host_msg["idx"], host_msg["w"]
    # float64 copies: numpy would otherwise add up the squares of a million float32 entries in float32
    U, V = np.asarray(host_msg["U"], dtype=np.float64), np.asarray(host_msg["V"], dtype=np.float64)
    s1 = float(sigma_gpu[0])
    assert (np.diff(idx) > 0).all()
    if idx.size == 0:
        return
    # unit-norm, mutually orthogonal atoms
    np.testing.assert_allclose(np.linalg.norm(U, axis=0), 1.0, atol=2e-5)
    np.testing.assert_allclose(np.linalg.norm(V, axis=0), 1.0, atol=2e-5)
    assert np.abs(U.T @ U - np.eye(idx.size)).max() < tol
    assert np.abs(V.T @ V - np.eye(idx.size)).max() < tol
    # each kept atom is a singular pair of G: G v = sigma u, G^T u = sigma v
    sig = np.asarray(sigma_gpu, dtype=np.float64)[idx]
    assert np.abs(G @ V - U * sig).max() < tol * s1
    assert np.abs(G.T @ U - V * sig).max() < tol * s1
    # weights are sigma / p
    np.testing.assert_allclose(w, sig / np.asarray(p_gpu, dtype=np.float64)[idx], rtol=1e-5)
