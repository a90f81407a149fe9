"""The layer sets of Section 6 (Table "datasets": ResNet-18 and VGG-11-BN on CIFAR-10) and its reshape of a
convolution gradient [x, y, k, k] into a matrix [x*y/2, 2*k*k], checked on the CPU against what the paper
prints and against the oracle."""
import numpy as np
import torch

import oracle
from paper_1806_04090_amd import inputs


def test_parameter_counts_match_the_table():
    # Table "datasets": 11,173k parameters for ResNet-18, 9,756k for VGG-11-BN.  Weights in the layer sets plus
    # what is not a matrix: one BN scale and shift per conv output channel, conv biases for VGG, FC biases.
    res_w = sum(x * y * k * k for x, y, k in inputs.RESNET18_CONVS) + sum(o * i for o, i in inputs.RESNET18_FCS)
    res_bn = 2 * sum(x for x, _, _ in inputs.RESNET18_CONVS)
    res_total = res_w + res_bn + sum(o for o, _ in inputs.RESNET18_FCS)
    assert res_w == inputs.RESNET18_ELEMENTS == 11_164_352
    assert res_total == inputs.RESNET18_PARAMETERS and res_total // 1000 == 11_173
    vgg_w = sum(x * y * k * k for x, y, k in inputs.VGG11BN_CONVS) + sum(o * i for o, i in inputs.VGG11BN_FCS)
    vgg_scalars = 3 * sum(x for x, _, _ in inputs.VGG11BN_CONVS) + sum(o for o, _ in inputs.VGG11BN_FCS)
    assert vgg_w + vgg_scalars == inputs.VGG11BN_PARAMETERS and inputs.VGG11BN_PARAMETERS // 1000 == 9_756


def test_reshape_is_a_view_of_the_same_memory():
    for convs, fcs, shapes in ((inputs.RESNET18_CONVS, inputs.RESNET18_FCS, inputs.RESNET18_SECTION6_SHAPES),
                               (inputs.VGG11BN_CONVS, inputs.VGG11BN_FCS, inputs.VGG11BN_SECTION6_SHAPES)):
        for (x, y, k), (rows, cols) in zip(convs, shapes):
            assert rows * cols == x * y * k * k and cols == 2 * k * k and rows == x * y // 2
            t = torch.arange(x * y * k * k).reshape(x, y, k, k)
            v = t.view(rows, cols)
            assert v.data_ptr() == t.data_ptr() and v.is_contiguous()
        assert list(shapes[len(convs):]) == list(fcs)
    # the standard view and the reshape hold the same elements
    assert sum(m * n for m, n in inputs.RESNET18_SECTION6_SHAPES) == sum(m * n for m, n in inputs.RESNET18_SHAPES)


def test_oracle_on_a_reshaped_gradient():
    # a [16, 8, 3, 3] gradient as out x in*k*k (16 x 72) and in the reshape (64 x 18): same Frobenius norm, so the
    # same sum of squared singular values; the reshape has 18 atoms instead of 16
    rng = np.random.default_rng(0)
    g = rng.standard_normal((16, 8, 3, 3))
    a, b = g.reshape(16, 72), g.reshape(64, 18)
    sa, _, _ = oracle.svd(a)
    sb, ub, vb = oracle.svd(b)
    assert sa.size == 16 and sb.size == 18
    np.testing.assert_allclose((sa ** 2).sum(), (g ** 2).sum(), rtol=1e-12)
    np.testing.assert_allclose((sb ** 2).sum(), (g ** 2).sum(), rtol=1e-12)
    np.testing.assert_allclose(sb, np.linalg.svd(b, compute_uv=False), rtol=1e-10)
    np.testing.assert_allclose((ub * sb) @ vb.T, b, atol=1e-12)
    # the estimator is unbiased in either view: sum_i p_i * (sigma_i / p_i) u_i v_i^T = G
    p = oracle.probabilities(sb, 3.0)
    np.testing.assert_allclose(p.sum(), 3.0, rtol=1e-12)
    mean = sum(p[i] * (sb[i] / p[i]) * np.outer(ub[:, i], vb[:, i]) for i in range(18))
    np.testing.assert_allclose(mean.reshape(16, 8, 3, 3), g, atol=1e-12)


def test_section6_generator_shapes_and_seed():
    mats = inputs.section6_layer_set(3, [(96, 18), (4096, 2), (10, 512)])
    again = inputs.section6_layer_set(3, [(96, 18), (4096, 2), (10, 512)])
    assert [m.shape for m in mats] == [(96, 18), (4096, 2), (10, 512)]
    assert all(m.dtype == np.float32 and m.flags.c_contiguous for m in mats)
    assert all(np.array_equal(x, y) for x, y in zip(mats, again))
