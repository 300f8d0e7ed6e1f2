"""Seeded synthetic inputs shared by the CPU reference and the GPU library's tests.

Holds no arithmetic of the method: only draws images, labels, parameter vectors and stress
gradients with numpy's counter-based Philox bit generator.  The recipe stands in for the
CIFAR-10 / ImageNet batches of the paper's experiments (same tensor shapes, value range and
class counts; pixel values i.i.d. uniform, labels uniform).
"""
import numpy as np

PURPOSE = dict(images=0, labels=1, weights=2, attack_init=3, quantizer=4, misc=5)


def _rng(config, purpose):
    return np.random.Generator(np.random.Philox(key=(int(config) << 32) + PURPOSE[purpose]))


def seed_for(config, purpose):
    """64-bit seed handed to dat_attack / dat_quantize for a given config and purpose."""
    return (int(config) << 32) + PURPOSE[purpose]


def images(config, B, H, W, C=3):
    """fp32 NHWC pixels, i.i.d. uniform on [0,1)."""
    return _rng(config, "images").random((B, H, W, C), dtype=np.float32)


def labels(config, B, num_classes):
    return _rng(config, "labels").integers(0, num_classes, size=B, dtype=np.int32)


def he_normal_params(config, offsets, fan_in, kind, residual_gamma=1.0):
    """Flat fp32 parameter vector: weights N(0, 2/fan_in); BN gamma = 1, beta = 0; biases = 0.

    `kind` per tensor: 0 conv weight, 1 conv bias, 2 BN gamma, 3 BN beta, 4 linear weight,
    5 linear bias, 6 gamma of the last BN of a residual branch (set to `residual_gamma`; values
    below 1 give the damped-branch initialisation common in large-batch training).
    """
    rng = _rng(config, "weights")
    d = int(offsets[-1])
    flat = np.zeros(d, np.float32)
    for t in range(len(kind)):
        lo, hi = int(offsets[t]), int(offsets[t + 1])
        if kind[t] in (0, 4):
            flat[lo:hi] = rng.standard_normal(hi - lo, dtype=np.float32) * np.float32(np.sqrt(2.0 / fan_in[t]))
        elif kind[t] == 2:
            flat[lo:hi] = 1.0
        elif kind[t] == 6:
            flat[lo:hi] = residual_gamma
    return flat


def perturbed_params(config, offsets, fan_in, kind, residual_gamma=1.0):
    """As he_normal_params but with non-trivial BN affine parameters and biases, so that
    tests see gradients flow through every parameter kind."""
    rng = _rng(config, "misc")
    flat = he_normal_params(config, offsets, fan_in, kind, residual_gamma)
    for t in range(len(kind)):
        lo, hi = int(offsets[t]), int(offsets[t + 1])
        if kind[t] in (2, 6):
            flat[lo:hi] *= 1.0 + 0.2 * rng.standard_normal(hi - lo, dtype=np.float32)
        elif kind[t] in (1, 3, 5):
            flat[lo:hi] = 0.1 * rng.standard_normal(hi - lo, dtype=np.float32)
    return flat


def stress_gradient(config, offsets):
    """Gradient-like vector: per-tensor N(0,1) * 10^U(-6,0) (layers differ by orders of
    magnitude), with one tensor all zero and one holding a single huge outlier."""
    rng = _rng(config, "quantizer")
    T = len(offsets) - 1
    g = np.zeros(int(offsets[-1]), np.float32)
    for t in range(T):
        lo, hi = int(offsets[t]), int(offsets[t + 1])
        g[lo:hi] = rng.standard_normal(hi - lo, dtype=np.float32) * np.float32(10.0 ** rng.uniform(-6, 0))
    if T >= 3:
        lo, hi = int(offsets[1]), int(offsets[2])
        g[lo:hi] = 0.0
        lo, hi = int(offsets[2]), int(offsets[3])
        if hi > lo:
            g[lo + (hi - lo) // 2] = 1.0e4
    return g


def ragged_offsets(config, T, max_len):
    """Tensor table with lengths that are not multiples of 4 or of the wavefront size."""
    rng = _rng(config, "misc")
    lens = rng.integers(1, max_len, size=T)
    lens[0] = 1
    if T > 1:
        lens[1] = 63
    if T > 2:
        lens[2] = 257
    return np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
