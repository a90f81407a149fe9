"""GPU parity: atomo_probabilities against the oracle's Algorithm 1."""
import numpy as np
import pytest

import oracle
from paper_1806_04090_amd import binding, inputs
from gpu_common import ctx, dev

pytestmark = pytest.mark.gpu


def run(lam, offsets, s):
    return binding.atomo_probabilities(ctx(), dev(np.asarray(lam, dtype=np.float32)), offsets, s).cpu().numpy()


def compare(lam32, p_gpu, s):
    want = oracle.probabilities(lam32.astype(np.float64), s)
    np.testing.assert_allclose(p_gpu, want, rtol=1e-6, atol=1e-12)
    assert ((want == 1) == (p_gpu == 1)).mean() > 0.999999 or np.abs(want - p_gpu).max() < 1e-6


def test_hand_examples_and_degenerate_segments():
    lam = np.array([4, 1, 1, 3, 2, 1, 10, 5, 1, 1, 0, 0, 0, 5, 0, 5, 0, 7], dtype=np.float32)
    offsets = [0, 3, 6, 10, 10, 13, 17, 18]
    p = run(lam, offsets, 2.0)
    want = [1, .5, .5, 1, 2 / 3, 1 / 3, 1, 5 / 7, 1 / 7, 1 / 7, 0, 0, 0, 1, 0, 1, 0, 1]
    np.testing.assert_allclose(p, want, rtol=1e-6)


@pytest.mark.parametrize("n", [1, 2, 31, 64, 65, 500, 2048])
def test_small_segments_sort_path(n):
    rng = np.random.default_rng(n)
    lam = (rng.standard_normal(n) * np.exp(2 * rng.standard_normal(n))).astype(np.float32)
    lam[rng.random(n) < 0.1] = 0
    for s in (0.5, 1.0, 3.0, n / 3 + 0.25, float(n), n + 2.0):
        compare(lam, run(lam, [0, n], s), s)


@pytest.mark.parametrize("n,kind", [(2049, "lognormal"), (10_000, "lognormal"), (100_003, "heavy"),
                                    (65_536, "ties"), (50_000, "equal"), (30_000, "zeros")])
def test_large_segments_histogram_path(n, kind):
    rng = np.random.default_rng(n)
    if kind == "lognormal":
        lam = rng.standard_normal(n) * np.exp(2 * rng.standard_normal(n))
    elif kind == "heavy":
        lam = inputs.flat_heavy_tail(1, n=n).astype(np.float64)
    elif kind == "ties":
        lam = rng.integers(-4, 5, size=n).astype(np.float64) * 0.25
    elif kind == "equal":
        lam = np.full(n, -0.37)
    else:
        lam = np.where(rng.random(n) < 0.001, rng.standard_normal(n), 0.0)
    lam = lam.astype(np.float32)
    nnz = int((lam != 0).sum())
    for s in (1.0, 17.5, n / 100, n / 7 + 0.5, nnz - 0.5, float(nnz), float(n), n + 10.0):
        if s <= 0:
            continue
        compare(lam, run(lam, [0, n], s), s)


def test_many_segments_mixed_sizes_and_unaligned_starts():
    rng = np.random.default_rng(5)
    sizes = [3, 700, 1, 5000, 64, 2049, 2048, 9, 12345]
    offsets = np.concatenate([[0], np.cumsum(sizes)]).tolist()
    lam = (rng.standard_normal(offsets[-1]) * np.exp(rng.standard_normal(offsets[-1]))).astype(np.float32)
    p = run(lam, offsets, 4.0)
    for a, b in zip(offsets[:-1], offsets[1:]):
        compare(lam[a:b], p[a:b], 4.0)


def test_quantisation_presets_closed_form():
    # Section 4: s = |g|_1/|g|_2 gives p = |g|/|g|_2 (1-bit QSGD); s = |g|_1/|g|_inf gives |g|/|g|_inf (TernGrad)
    rng = np.random.default_rng(6)
    g = rng.standard_normal(40_000).astype(np.float32)
    a = np.abs(g.astype(np.float64))
    for norm in (np.sqrt((a ** 2).sum()), a.max()):
        p = run(g, [0, g.size], a.sum() / norm)
        np.testing.assert_allclose(p, np.minimum(1.0, a / norm), rtol=2e-6, atol=1e-12)


@pytest.mark.parametrize("n", [11, 1635, 2048, 2049, 60_000])
def test_wide_dynamic_range(n):
    # magnitudes from 1e-30 to 1e30 in one segment: the tail sums behind the forced atoms must keep the small
    # values (sort path up to 2048 atoms, histogram path above)
    rng = np.random.default_rng(n)
    lam = rng.choice(np.array([0.0, 1.0, 1.0000001, 2.0, 1e-30, 1e30], dtype=np.float32), n)
    lam[:6] = [1e30, 2.0, 1.0, 1e-30, 0.0, 1.0000001]
    for s in (0.5, float((lam == np.float32(1e30)).sum()) + 2.0, n / 3.0):
        p = run(lam, [0, n], s)
        want = oracle.probabilities(lam.astype(np.float64), s)
        np.testing.assert_allclose(p, want, rtol=1e-6, atol=1e-44)
