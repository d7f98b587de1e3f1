"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds no arithmetic of the method: only random draws with the shapes and value
distributions of the paper's workload (3x224x224 images standing in for ImageNet,
1000 classes, per-worker minibatch 32; He-normal convolution filters, BN scale 1 and
shift 0, FC weights N(0, 0.01^2) as in the recipe the paper builds on).  All arrays are
float32 in logical NCHW / KCRS order; draw order is fixed: activations first, then
parameters in table order, then upstream gradients or labels.
"""
import numpy as np


def rng(seed):
    return np.random.default_rng(seed)


def normal(g, shape, std=1.0, mean=0.0):
    return (g.standard_normal(shape, dtype=np.float32) * np.float32(std) + np.float32(mean)).astype(np.float32)


def he_normal(g, shape):
    """shape = (K, C, R, S); std = sqrt(2 / (C*R*S))."""
    fan_in = int(np.prod(shape[1:]))
    return normal(g, shape, std=float(np.sqrt(2.0 / fan_in)))


def labels(g, n, classes=1000):
    return g.integers(0, classes, size=n, dtype=np.int32)


def params(g, table, perturb_bn=False):
    """table: [(name, shape, kind)], kind in conv_w, bn_g, bn_b, fc_w, fc_b.  Returns {name: float32 array}.
    perturb_bn draws BN scale ~ N(1, 0.1^2) and shift ~ N(0, 0.1^2) instead of the constants 1 and 0."""
    out = {}
    for name, shape, kind in table:
        if kind == "conv_w":
            out[name] = he_normal(g, shape)
        elif kind == "bn_g":
            out[name] = normal(g, shape, 0.1, 1.0) if perturb_bn else np.ones(shape, np.float32)
        elif kind == "bn_b":
            out[name] = normal(g, shape, 0.1) if perturb_bn else np.zeros(shape, np.float32)
        elif kind == "fc_w":
            out[name] = normal(g, shape, 0.01)
        elif kind == "fc_b":
            out[name] = np.zeros(shape, np.float32)
        else:
            raise ValueError(kind)
    return out


def fp32_bit_patterns(g, count):
    """Random 32-bit patterns viewed as float32: exercises every exponent, subnormals, infinities and NaNs."""
    return g.integers(0, 2**32, size=count, dtype=np.uint64).astype(np.uint32).view(np.float32)


def gradient_like(g, count):
    """Values with the spread of real gradients: N(0,1) times a log-uniform magnitude in [1e-9, 1e2]."""
    mag = np.exp(g.uniform(np.log(1e-9), np.log(1e2), size=count)).astype(np.float32)
    return (g.standard_normal(count, dtype=np.float32) * mag).astype(np.float32)
