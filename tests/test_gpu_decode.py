"""GPU parity: atomo_decode fed oracle-made messages."""
import numpy as np
import pytest
import torch

import oracle
from paper_1806_04090_amd import binding
from gpu_common import ctx, dev

pytestmark = pytest.mark.gpu


def make_msg(rng, rows, cols, k, capacity):
    host = {"w": rng.standard_normal(k), "U": rng.standard_normal((rows, k)), "V": rng.standard_normal((cols, k))}
    m = binding.alloc_svd_message(rows, cols, capacity, "cuda")
    m.count.fill_(k)
    m.idx[:k] = torch.arange(k, dtype=torch.int32)
    m.w[:k] = dev(host["w"].astype(np.float32))
    m.U[:k] = dev(host["U"].T.astype(np.float32))
    m.V[:k] = dev(host["V"].T.astype(np.float32))
    host = {key: val.astype(np.float32).astype(np.float64) for key, val in host.items()}
    return m, host


@pytest.mark.parametrize("rows,cols,ks", [(1, 1, [1]), (5, 7, [3]), (64, 576, [2]), (70, 300, [0, 4, 1]),
                                          (130, 1030, [3, 3, 2, 5]), (512, 4608, [3]), (10, 512, [48])])
def test_svd_decode_matches_oracle(rows, cols, ks):
    rng = np.random.default_rng(rows * 31 + cols)
    pairs = [make_msg(rng, rows, cols, k, max(k, 1) + 2) for k in ks]
    scale = 1.0 / len(ks)
    out = binding.atomo_decode(ctx(), [m for m, _ in pairs], scale=scale).cpu().numpy()
    want = oracle.decode_svd([h for _, h in pairs], rows, cols, scale=scale)
    assert np.linalg.norm(out - want) <= 1e-5 * max(np.linalg.norm(want), 1e-30)
    np.testing.assert_allclose(out, want, rtol=0, atol=1e-5 * max(np.abs(want).max(), 1e-30))


@pytest.mark.parametrize("rows,cols,capacity,ks", [(40, 130, 100, [7, 0, 99, 100, 1, 33, 2, 2, 2, 50, 5, 64]),   # batches of 5 messages
                                                   (96, 70, 512, [512, 3]),                                     # the atom list is staged in two pieces
                                                   (600, 600, 600, [600]),                                      # every atom of a 600 x 600 matrix kept (p = 1)
                                                   (130, 2048, 130, [130, 129, 1]),
                                                   (33, 33, 6, [5] * 90)])                                      # 85 messages per batch, then 5
def test_svd_decode_many_messages_across_batches(rows, cols, capacity, ks):
    rng = np.random.default_rng(len(ks) * 7 + rows)
    pairs = [make_msg(rng, rows, cols, k, capacity) for k in ks]
    out = binding.atomo_decode(ctx(), [m for m, _ in pairs], scale=0.5).cpu().numpy()
    want = oracle.decode_svd([h for _, h in pairs], rows, cols, scale=0.5)
    assert np.linalg.norm(out - want) <= 1e-5 * max(np.linalg.norm(want), 1e-30)


def test_svd_decode_into_strided_output_and_batch():
    rng = np.random.default_rng(1)
    m1, h1 = make_msg(rng, 33, 50, 2, 4)
    m2, h2 = make_msg(rng, 70, 20, 3, 4)
    big = torch.full((33, 64), 7.0, device="cuda")
    binding.atomo_decode(ctx(), [m1], out=big[:, 3:53])
    got = big.cpu().numpy()
    np.testing.assert_allclose(got[:, 3:53], oracle.decode_svd([h1], 33, 50), rtol=1e-5, atol=1e-5)
    assert (got[:, :3] == 7).all() and (got[:, 53:] == 7).all()
    outs = binding.atomo_decode_svd_batch(ctx(), [[m1], [m2]])
    np.testing.assert_allclose(outs[0].cpu().numpy(), oracle.decode_svd([h1], 33, 50), rtol=1e-5, atol=1e-5)
    np.testing.assert_allclose(outs[1].cpu().numpy(), oracle.decode_svd([h2], 70, 20), rtol=1e-5, atol=1e-5)


def test_entrywise_decode_matches_oracle():
    rng = np.random.default_rng(2)
    n = 10_007
    msgs, hosts = [], []
    for k in (0, 1, 500):
        idx = np.sort(rng.choice(n, size=k, replace=False))
        val = rng.standard_normal(k).astype(np.float32)
        m = binding.alloc_entrywise_message(n, max(k, 1), "cuda")
        m.count.fill_(k)
        if k:
            m.idx[:k] = dev(idx.astype(np.uint32).view(np.int32))
            m.val[:k] = dev(val)
        msgs.append(m); hosts.append({"idx": idx, "val": val.astype(np.float64)})
    out = binding.atomo_decode(ctx(), msgs, scale=0.5).cpu().numpy()
    np.testing.assert_allclose(out, oracle.decode_entrywise(hosts, n, scale=0.5), rtol=1e-6, atol=1e-9)


def test_matrix_core_rate_probe_returns_a_plausible_figure():
    # the measurement helper of bench.py: between a tenth of and the whole published fp32 matrix-core peak
    rate = ctx().measure_mfma_fp32()
    assert 15.0 < rate < 160.0
