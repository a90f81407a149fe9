"""Seeded random sweep of atomo_encode_svd over shapes of all three kinds (thin, blocked, Gram-space) and over
spectra that stress different parts of the iteration: pure noise at odd scales, exact low rank, graded, clustered,
duplicated rows, zero rows and columns.  sigma against LAPACK in fp64 (tolerance of the other SVD tests, with the
fp32 floor of 32 ulp of sigma_1 for values that are zero in exact arithmetic), p against the oracle's Algorithm 1
on the GPU's sigma, the mask bit-exact, kept atoms through the singular-pair properties."""
import numpy as np
import pytest
import torch

import oracle
from paper_1806_04090_amd import binding, inputs
from gpu_common import ctx, dev, sigma_tolerance_ok, check_svd_message_against_matrix

pytestmark = pytest.mark.gpu

FLOOR = 32 * 2.0 ** -24 * 1.01


def make(rng, kind, m, n):
    r = min(m, n)
    if kind == "noise":
        return rng.standard_normal((m, n)) * 10.0 ** rng.uniform(-6, 2)
    if kind == "lowrank":
        k = int(rng.integers(1, max(2, r // 4)))
        return (rng.standard_normal((m, k)) * (0.5 ** np.arange(k))) @ rng.standard_normal((k, n))
    if kind == "lownoise":
        return inputs.low_rank_plus_noise(rng, m, n, 0.5 ** np.arange(int(rng.integers(1, 9))), 10.0 ** rng.uniform(-4, -1))
    u, _ = np.linalg.qr(rng.standard_normal((m, r)))
    v, _ = np.linalg.qr(rng.standard_normal((n, r)))
    if kind == "graded":
        return (u * 10.0 ** (-rng.uniform(1, 4) * np.arange(r) / max(r - 1, 1))) @ v.T
    if kind == "cluster":
        return (u * (np.where(rng.random(r) < 0.5, 1.0, 0.3) * (1 + 1e-6 * rng.standard_normal(r)))) @ v.T
    g = rng.standard_normal((m, n))
    if kind == "duprows":
        g[m // 2:] = g[:m - m // 2]
    elif kind == "zeros":
        g[:, rng.random(n) < 0.5] = 0
        g[rng.random(m) < 0.3] = 0
    else:                                                        # "scaled": far from 1, inside the fp32 range
        g *= 10.0 ** rng.choice([-25, -15, 12, 17])
    return g


KINDS = ["noise", "lowrank", "lownoise", "graded", "cluster", "duprows", "zeros", "scaled"]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_shapes_and_spectra(seed):
    rng = np.random.default_rng(1000 + seed)
    c = ctx()
    for it in range(32):
        kind = KINDS[it % len(KINDS)]
        cls = (it // len(KINDS)) % 4
        if cls == 0:
            m, n = int(rng.integers(1, 33)), int(rng.integers(1, 5000))
        elif cls == 1:
            m, n = int(rng.integers(33, 200)), int(rng.integers(33, 1500))
        elif cls == 2:
            m, n = int(rng.integers(200, 481)), int(rng.integers(200, 1200))
        else:
            m, n = int(rng.integers(481, 640)), int(rng.integers(481, 900))
        if rng.random() < 0.5:
            m, n = n, m
        G = np.ascontiguousarray(make(rng, kind, m, n), dtype=np.float32)
        r = min(m, n)
        s = float(rng.uniform(1, min(r, 8) + 0.5))
        sig = torch.zeros(r, device="cuda")
        p = torch.zeros(r, device="cuda")
        msg = binding.alloc_svd_message(m, n, r, "cuda")
        binding.atomo_encode_svd(c, [dev(G)], s, it, 7, msgs=[msg], sigma_out=sig, p_out=p, max_sweeps=32)
        where = f"seed {seed} case {it} {kind} {m}x{n} s={s:.2f}"
        assert c.status()[0] == 0, where
        ref = np.linalg.svd(G.astype(np.float64), compute_uv=False)
        sg, pg = sig.cpu().numpy(), p.cpu().numpy()
        at_floor = (sg <= FLOOR * ref[0]) & (ref <= FLOOR * ref[0])
        assert (sigma_tolerance_ok(sg, ref) | at_floor).all(), where
        np.testing.assert_allclose(pg, oracle.probabilities(sg.astype(np.float64), s), rtol=1e-5, atol=1e-9, err_msg=where)
        h = msg.to_host()
        assert np.array_equal(h["idx"], np.flatnonzero(oracle.bernoulli_mask(pg, it, 7))), where
        check_svd_message_against_matrix(G.astype(np.float64), h, sg, pg)


def test_budget_above_the_rank_keeps_the_real_atoms_only():
    # rank 2 in 7 columns, budget 6: the five singular values that are zero in exact arithmetic come out as 0 with
    # p = 0; the two real atoms have p = 1 (KKT appendix: s >= number of nonzeros) and reproduce the matrix
    rng = np.random.default_rng(9)
    for shape in [(3359, 7), (10, 57), (320, 148), (600, 520)]:
        G = (rng.standard_normal((shape[0], 2)) @ rng.standard_normal((2, shape[1]))).astype(np.float32)
        r = min(shape)
        sig = torch.zeros(r, device="cuda")
        p = torch.zeros(r, device="cuda")
        msg = binding.alloc_svd_message(*shape, r, "cuda")
        binding.atomo_encode_svd(ctx(), [dev(G)], 6.0, 1, 0, msgs=[msg], sigma_out=sig, p_out=p)
        assert ctx().status()[0] == 0
        h = msg.to_host()
        assert h["count"] == 2 and list(h["idx"]) == [0, 1]
        assert (sig[2:] == 0).all() and (p[2:] == 0).all() and (p[:2] == 1).all()
        check_svd_message_against_matrix(G.astype(np.float64), h, sig.cpu().numpy(), p.cpu().numpy())
        out = binding.atomo_decode(ctx(), [msg]).cpu().numpy()
        assert np.linalg.norm(out - G) <= 1e-5 * np.linalg.norm(G)
