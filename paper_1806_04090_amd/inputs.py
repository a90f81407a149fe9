"""Seeded synthetic gradients.  No ATOMO arithmetic lives here.

The paper measures on gradients of ResNet-18 / VGG-11-BN trained on CIFAR-10 and SVHN
(Section 6, Table "datasets").  Those gradients are not available; the generators below
stand in for them: they take the layer shapes and the parameter count of those models and
the "few dominant singular values over a noise floor" structure of Fig. 1.

Everything is drawn in float64 from ``numpy.random.default_rng(seed)`` and rounded to
float32 once; the same float32 array feeds the HIP library and (upcast) the oracle.
This module is the only code the two sides share.
"""
from __future__ import annotations

import numpy as np

# ResNet-18 (CIFAR-10 sizing) weight gradients as out x (in*k*k) matrices, in network order.
RESNET18_SHAPES = (
    [(64, 27)]
    + [(64, 576)] * 4
    + [(128, 576)] + [(128, 1152)] * 3 + [(128, 64)]
    + [(256, 1152)] + [(256, 2304)] * 3 + [(256, 128)]
    + [(512, 2304)] + [(512, 4608)] * 3 + [(512, 256)]
    + [(10, 512)]
)
RESNET18_ELEMENTS = sum(m * n for m, n in RESNET18_SHAPES)        # 11,164,352
RESNET18_PARAMETERS = 11_173_962                                   # with the 9,610 BN / bias scalars

# Convolution weights [out, in, k, k] of the two CIFAR-10 models of Table "datasets", in network order, and their
# fully connected layers [out, in].
RESNET18_CONVS = (
    [(64, 3, 3)] + [(64, 64, 3)] * 4
    + [(128, 64, 3)] + [(128, 128, 3)] * 3 + [(128, 64, 1)]
    + [(256, 128, 3)] + [(256, 256, 3)] * 3 + [(256, 128, 1)]
    + [(512, 256, 3)] + [(512, 512, 3)] * 3 + [(512, 256, 1)]
)
RESNET18_FCS = [(10, 512)]
VGG11BN_CONVS = [(64, 3, 3), (128, 64, 3), (256, 128, 3), (256, 256, 3),
                 (512, 256, 3), (512, 512, 3), (512, 512, 3), (512, 512, 3)]
VGG11BN_FCS = [(512, 512), (512, 512), (10, 512)]
VGG11BN_PARAMETERS = 9_756_426                                     # with the BN / bias scalars


def section6_reshape(convs, fcs):
    """Matrix shapes under the reshape of Section 6: a conv gradient [x, y, k, k] is viewed as
    [x*y/2, 2*k*k] (same memory, no copy); fully connected layers stay [out, in]."""
    return [(x * y // 2, 2 * k * k) for (x, y, k) in convs] + list(fcs)


RESNET18_SECTION6_SHAPES = section6_reshape(RESNET18_CONVS, RESNET18_FCS)
VGG11BN_SECTION6_SHAPES = section6_reshape(VGG11BN_CONVS, VGG11BN_FCS)


def _orthonormal(rng: np.random.Generator, dim: int, k: int) -> np.ndarray:
    """dim x k matrix with orthonormal columns: Q factor of a Gaussian matrix."""
    q, _ = np.linalg.qr(rng.standard_normal((dim, k)))
    return q


def low_rank_plus_noise(rng: np.random.Generator, m: int, n: int, sigmas, noise_std: float) -> np.ndarray:
    """sum_k sigmas[k] u_k v_k^T + N(0, noise_std^2), float32, C-contiguous."""
    sigmas = np.asarray(sigmas, dtype=np.float64)
    k = min(len(sigmas), m, n)
    u = _orthonormal(rng, m, k)
    v = _orthonormal(rng, n, k)
    x = (u * sigmas[:k]) @ v.T
    x += noise_std * rng.standard_normal((m, n))
    return np.ascontiguousarray(x, dtype=np.float32)


def single_conv_layer(seed: int = 0) -> np.ndarray:
    """One 64 x 576 gradient (3x3 conv, 64 -> 64): rank-4 signal 1, .5, .25, .125 plus N(0, 0.01^2)."""
    rng = np.random.default_rng(seed)
    return low_rank_plus_noise(rng, 64, 576, [1.0, 0.5, 0.25, 0.125], 0.01)


def resnet18_layer_set(seed: int = 0, shapes=RESNET18_SHAPES):
    """The 21 ResNet-18 matrices: rank-8 geometric signal 0.5^k (k = 0..7) plus N(0, 1e-3^2)."""
    rng = np.random.default_rng(seed)
    sig = 0.5 ** np.arange(8)
    return [low_rank_plus_noise(rng, m, n, sig, 1e-3) for (m, n) in shapes]


def section6_layer_set(seed: int = 0, shapes=RESNET18_SECTION6_SHAPES):
    """One matrix per layer in the Section 6 reshape: rank-min(8, cols, rows) geometric signal 0.5^k plus
    N(0, 1e-3^2), generated directly in the reshaped view."""
    rng = np.random.default_rng(seed)
    sig = 0.5 ** np.arange(8)
    return [low_rank_plus_noise(rng, m, n, sig, 1e-3) for (m, n) in shapes]


def vgg_deep_conv_batch(seed: int = 0, batch: int = 64, m: int = 512, n: int = 4608):
    """`batch` matrices m x n: rank-16 signal with sigma_k ~ U(0.1, 1) plus N(0, 1e-2^2)."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(batch):
        sig = rng.uniform(0.1, 1.0, size=16)
        out.append(low_rank_plus_noise(rng, m, n, sig, 1e-2))
    return out


def flat_heavy_tail(seed: int = 0, n: int = RESNET18_PARAMETERS, std: float = 1e-3,
                    heavy_fraction: float = 1e-3, heavy_scale: float = 100.0) -> np.ndarray:
    """Flat gradient N(0, std^2) with floor(n * heavy_fraction) distinct random entries multiplied by heavy_scale."""
    rng = np.random.default_rng(seed)
    g = std * rng.standard_normal(n)
    n_heavy = int(n * heavy_fraction)
    if n_heavy:
        pos = rng.choice(n, size=n_heavy, replace=False)
        g[pos] *= heavy_scale
    return g.astype(np.float32)


def worker_stream(worker: int, layer: int) -> int:
    """Philox stream id of layer `layer` of data-parallel worker `worker`."""
    return (worker << 32) | layer
