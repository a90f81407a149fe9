"""GPU parity for the reshape of Section 6: a conv gradient [x, y, k, k] viewed as [x*y/2, 2*k*k].

Those matrices have 18 columns (3x3 kernels) or 2 (1x1) and thousands of rows; the library takes them
through a path of its own (whole r x r problem in one workgroup, r <= 32).  Same bar as the other SVD
tests: sigma and p value by value, mask bit-exact given the GPU's p, vectors through the singular
pairs, decode against the oracle's decode of the same message."""
import numpy as np
import pytest
import torch

import oracle
from paper_1806_04090_amd import binding, inputs
from gpu_common import ctx, dev, sigma_tolerance_ok, check_svd_message_against_matrix
from test_gpu_svd import encode, full_parity

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape", [(96, 18), (2048, 18), (4096, 2), (1024 + 37, 18), (3000, 32), (5000, 31), (700, 7),
                                   (18, 2048), (2, 4096), (27, 1500), (257, 1), (1, 257)])
def test_thin_shapes_against_the_oracle(shape):
    rng = np.random.default_rng(shape[0] * 131 + shape[1])
    G = inputs.low_rank_plus_noise(rng, shape[0], shape[1], [1.0, 0.5, 0.25, 0.1], 0.01)
    r = min(shape)
    msgs, per, status, sweeps = encode([G], 3.0, 5, stream_base=9, capacity=r)
    assert status == 0 and ctx().svd_sweeps(1)[0] <= 3
    h = full_parity(G, 3.0, 5, 9, msgs[0], *per[0])
    out = binding.atomo_decode(ctx(), msgs).cpu().numpy()
    want = oracle.decode_svd([h], *shape)
    assert np.linalg.norm(out - want) <= 1e-5 * max(np.linalg.norm(want), 1e-30)


def test_section6_resnet18_layers_in_one_batch():
    # the small and medium layers of the set, all in one call (the large ones differ only in the row count)
    shapes = [s for s in inputs.RESNET18_SECTION6_SHAPES if s[0] <= 16384]
    mats = inputs.section6_layer_set(1, shapes)
    msgs, per, status, sweeps = encode(mats, 3.0, 2, stream_base=40)
    assert status == 0
    for j, G in enumerate(mats):
        full_parity(G, 3.0, 2, 40 + j, msgs[j], *per[j])
    groups = [[m] for m in msgs]
    outs = binding.atomo_decode_svd_batch(ctx(), groups)
    for j, (m, n) in enumerate(shapes):
        want = oracle.decode_svd([msgs[j].to_host()], m, n)
        assert np.linalg.norm(outs[j].cpu().numpy() - want) <= 1e-5 * max(np.linalg.norm(want), 1e-30)


def test_largest_layer_shape_sigma_and_pairs():
    # 131072 x 18 (a 512 -> 512 3x3 convolution): sigma against LAPACK in fp64, kept atoms through their pairs
    G = inputs.section6_layer_set(4, [(131072, 18)])[0]
    msgs, per, status, sweeps = encode([G], 3.0, 8)
    assert status == 0
    sig_ref = np.linalg.svd(G.astype(np.float64), compute_uv=False)
    assert sigma_tolerance_ok(per[0][0], sig_ref).all()
    np.testing.assert_allclose(per[0][1], oracle.probabilities(sig_ref, 3.0), rtol=1e-4, atol=1e-9)
    h = msgs[0].to_host()
    mask = oracle.bernoulli_mask(per[0][1], 8, 0)
    assert np.array_equal(h["idx"], np.flatnonzero(mask))
    check_svd_message_against_matrix(G.astype(np.float64), h, *per[0])


def test_padded_rows_and_a_mixed_batch():
    # a tall matrix whose rows are padded (ld > cols) is copied first; thin, blocked and Gram-space matrices together
    rng = np.random.default_rng(77)
    base = inputs.low_rank_plus_noise(rng, 900, 24, [1.0, 0.4, 0.2], 0.01)
    padded = torch.zeros(900, 40, dtype=torch.float32, device="cuda")[:, :24]
    padded.copy_(torch.from_numpy(base))
    assert padded.stride(0) == 40
    others = inputs.resnet18_layer_set(5, shapes=[(64, 576), (2048, 18), (512, 600)])
    c = ctx()
    mats = [padded] + [dev(g) for g in others]
    host = [base] + others
    total = sum(min(g.shape) for g in host)
    sigma = torch.zeros(total, device="cuda")
    p = torch.zeros(total, device="cuda")
    msgs = binding.atomo_encode_svd(c, mats, 3.0, 21, 0, sigma_out=sigma, p_out=p)
    assert c.status()[0] == 0
    offs = np.concatenate([[0], np.cumsum([min(g.shape) for g in host])])
    for j, G in enumerate(host):
        full_parity(G, 3.0, 21, j, msgs[j], sigma[offs[j]:offs[j + 1]].cpu().numpy(), p[offs[j]:offs[j + 1]].cpu().numpy())


def test_thin_graded_spectrum_and_rank_deficiency():
    rng = np.random.default_rng(5)
    # singular values over five decades, to the same tolerance as everywhere (floored at 1e-3 sigma_1)
    m, n = 4000, 12
    u, _ = np.linalg.qr(rng.standard_normal((m, n)))
    v, _ = np.linalg.qr(rng.standard_normal((n, n)))
    sig = 10.0 ** -np.linspace(0, 5, n)
    graded = np.ascontiguousarray((u * sig) @ v.T, dtype=np.float32)
    # rank 3 in 18 columns, and an all-zero matrix
    low = inputs.low_rank_plus_noise(rng, 3000, 18, [1.0, 0.5, 0.25], 0.0)
    zero = np.zeros((600, 18), dtype=np.float32)
    msgs, per, status, sweeps = encode([graded, low, zero], 3.0, 3, capacity=12)
    assert status == 0
    ref = np.linalg.svd(graded.astype(np.float64), compute_uv=False)
    assert sigma_tolerance_ok(per[0][0], ref).all(), float(np.abs(per[0][0] - ref).max())
    check_svd_message_against_matrix(graded.astype(np.float64), msgs[0].to_host(), *per[0])
    ref_low = np.linalg.svd(low.astype(np.float64), compute_uv=False)
    assert sigma_tolerance_ok(per[1][0][:3], ref_low[:3]).all()
    assert np.abs(per[1][0][3:]).max() <= 32 * 2.0 ** -24 * 1.01   # rounding residue, below the fp32 floor of the rows
    assert (per[2][0] == 0).all() and msgs[2].to_host()["count"] == 0
    check_svd_message_against_matrix(low.astype(np.float64), msgs[1].to_host(), *per[1])


def test_thin_pass_count_is_reported_and_limited():
    G = inputs.section6_layer_set(2, [(2048, 18)])[0]
    msgs, per, status, sweeps = encode([G], 3.0, 1)
    assert status == 0 and ctx().svd_sweeps(1)[0] in (1, 2)       # r x r problems solved
    # max_sweeps = 1 allows the thin path two passes, i.e. one rotation and the check after it
    msgs, per, status, sweeps = encode([G], 3.0, 1, max_sweeps=1)
    assert ctx().svd_sweeps(1)[0] == 1
    assert status in (0, binding.ATOMO_ENOCONV)


@pytest.mark.parametrize("shape", [(300_001, 18), (2, 700_000)])
def test_more_than_131072_positions(shape):
    # beyond 128 chunks of 1024 positions the chunks grow instead: several blocks per wave and chunk
    rng = np.random.default_rng(shape[0])
    G = inputs.low_rank_plus_noise(rng, shape[0], shape[1], [1.0, 0.5], 1e-3)
    msgs, per, status, sweeps = encode([G], 3.0, 1, capacity=min(shape))
    assert status == 0
    ref = np.linalg.svd(G.astype(np.float64), compute_uv=False)
    assert sigma_tolerance_ok(per[0][0], ref).all()
    h = msgs[0].to_host()
    assert np.array_equal(h["idx"], np.flatnonzero(oracle.bernoulli_mask(per[0][1], 1, 0)))
    check_svd_message_against_matrix(G.astype(np.float64), h, *per[0])
    out = binding.atomo_decode(ctx(), msgs).cpu().numpy()
    want = oracle.decode_svd([h], *shape)
    assert np.linalg.norm(out - want) <= 1e-5 * max(np.linalg.norm(want), 1e-30)
