"""Seeded synthetic inputs and the benchmark layer shapes.

This module serves both the CPU oracle's callers and the HIP library's callers
and holds none of the method's arithmetic: it only names layer shapes and draws
random tensors.  The shapes stand in for the paper's benchmark set (Section VI:
convolutions taken from AlexNet, NiN and GoogLeNetV1 at several batch sizes,
whose list the paper does not print); every tensor is synthetic.
"""
from collections import namedtuple

import numpy as np

# One forward-convolution problem.  dist_in: "u01" uniform[0,1) or "u11"
# uniform[-1,1); dist_filt: "n001" normal(0, std 0.01) or "u11"; dist_bias:
# "zero" (a real all-zero array), "u01b" uniform[-0.1,0.1) or "none" (NULL).
Layer = namedtuple("Layer", "name C H W K R S stride pad dist_in dist_filt dist_bias")

BASE_SEED = 160600094

TOY = Layer("toy3x3", 3, 32, 32, 16, 3, 3, 1, 1, "u11", "u11", "u01b")
CONV1 = Layer("conv1_11x11s4", 3, 227, 227, 96, 11, 11, 4, 0, "u01", "n001", "zero")
CONV2 = Layer("conv2_5x5", 96, 27, 27, 256, 5, 5, 1, 2, "u01", "n001", "u01b")
CONV3 = Layer("conv3_3x3", 256, 13, 13, 384, 3, 3, 1, 1, "u01", "n001", "u01b")
CONV4 = Layer("conv4_3x3", 384, 13, 13, 384, 3, 3, 1, 1, "u01", "n001", "u01b")
CONV5 = Layer("conv5_3x3", 384, 13, 13, 256, 3, 3, 1, 1, "u01", "n001", "u01b")
PW_A = Layer("pw_480x14_192", 480, 14, 14, 192, 1, 1, 1, 0, "u01", "n001", "u01b")
PW_B = Layer("pw_832x7_384", 832, 7, 7, 384, 1, 1, 1, 0, "u01", "n001", "u01b")
PW_C = Layer("pw_192x28_64", 192, 28, 28, 64, 1, 1, 1, 0, "u01", "n001", "u01b")
RED3 = Layer("red3x3_96x28_128", 96, 28, 28, 128, 3, 3, 1, 1, "u01", "n001", "u01b")
RED5 = Layer("red5x5_16x28_32", 16, 28, 28, 32, 5, 5, 1, 2, "u01", "n001", "u01b")

# The groups follow the five benchmark configurations.
CONFIG_TOY = [TOY]
CONFIG_FIRST = [CONV1]
CONFIG_MIDDLE = [CONV2, CONV3, CONV4, CONV5]
CONFIG_POINTWISE = [PW_A, PW_B, PW_C, RED3, RED5]
STACK = [CONV1, CONV2, CONV3, CONV4, CONV5]   # 3x3/s2 max-pool after conv1 and conv2
STACK_POOL_AFTER = (0, 1)
# Layers that a 3x3 / step-2 max pooling follows in the network the stack is cut from
# (swept through the convolution + pooling call by the tuner).
POOLED_LAYERS = [CONV1, CONV2, CONV5]
ALL_LAYERS = CONFIG_TOY + CONFIG_FIRST + CONFIG_MIDDLE + CONFIG_POINTWISE

# Square single-precision matrix products at the sizes of the paper's two SGEMM
# tables (Section V), each written as the pointwise layer it runs as:
# C[M x N] = A[M x K] * B[K x N]  <->  filters A, one image B of K channels, 1 x N pixels.
SGEMM_SIZES = (128, 256, 384, 512, 768, 1024, 1536, 2048)
# A is drawn like filters (normal, std 0.01) and B like activations (uniform[0,1)), so that
# the convolution tolerance, which is absolute near zero, means the same thing here.
SGEMM_LAYERS = [Layer("sgemm_%d" % n, n, 1, n, n, 1, 1, 1, 0, "u01", "n001", "none") for n in SGEMM_SIZES]

# Further layer shapes of the same three networks (and a few shapes outside them:
# stride-2 pointwise, non-square kernels) that the selection table does NOT list.
# They exercise the selection heuristic and the generic tiles on unseen shapes.
_E = lambda name, C, H, K, R, S, stride, pad, W=None: Layer(name, C, H, W or H, K, R, S, stride, pad,
                                                            "u01", "n001", "u01b")
EXTRA_LAYERS = [
    _E("x_1x1_192x28_96", 192, 28, 96, 1, 1, 1, 0),
    _E("x_3x3_128x28_192", 128, 28, 192, 3, 3, 1, 1),
    _E("x_5x5_32x28_96", 32, 28, 96, 5, 5, 1, 2),
    _E("x_3x3_112x14_224", 112, 14, 224, 3, 3, 1, 1),
    _E("x_5x5_32x14_128", 32, 14, 128, 5, 5, 1, 2),
    _E("x_3x3_192x7_384", 192, 7, 384, 3, 3, 1, 1),
    _E("x_1x1_96x55_96", 96, 55, 96, 1, 1, 1, 0),
    _E("x_3x3_384x13_1024", 384, 13, 1024, 3, 3, 1, 1),
    _E("x_1x1_1024x6_1000", 1024, 6, 1000, 1, 1, 1, 0),
    _E("x_7x7s2_3x224_64", 3, 224, 64, 7, 7, 2, 3),
    _E("x_3x3_64x56_192", 64, 56, 192, 3, 3, 1, 1),
    _E("x_1x1s2_256x28_512", 256, 28, 512, 1, 1, 2, 0),
    _E("x_1x7_128x17_128", 128, 17, 128, 1, 7, 1, 0),
    _E("x_7x1_128x17_128", 128, 17, 128, 7, 1, 1, 0),
    _E("x_3x3s2_96x27_160", 96, 27, 160, 3, 3, 2, 0),
    _E("x_5x5_13x20x31_50", 13, 20, 50, 5, 5, 1, 2, W=31),
]
BY_NAME = {l.name: l for l in ALL_LAYERS + SGEMM_LAYERS + EXTRA_LAYERS}


def _draw(rng, dist, shape):
    if dist == "u01":
        return rng.random(shape, dtype=np.float32)
    if dist == "u11":
        return (rng.random(shape, dtype=np.float32) * 2.0 - 1.0).astype(np.float32)
    if dist == "n001":
        return (rng.standard_normal(shape, dtype=np.float32) * np.float32(0.01)).astype(np.float32)
    if dist == "u01b":
        return ((rng.random(shape, dtype=np.float32) * 2.0 - 1.0)
                * np.float32(0.1)).astype(np.float32)
    if dist == "zero":
        return np.zeros(shape, dtype=np.float32)
    raise ValueError(dist)


def layer_seed(layer, N):
    """Seed of one (layer, batch) problem: base + 1000*index + N."""
    idx = [l.name for l in ALL_LAYERS + SGEMM_LAYERS + EXTRA_LAYERS].index(layer.name)
    return BASE_SEED + 1000 * idx + N


def make_layer_inputs(layer, N, seed=None):
    """(in[N,C,H,W], filt[K,C,R,S], bias[K] or None), fp32, drawn in that order."""
    rng = np.random.default_rng(layer_seed(layer, N) if seed is None else seed)
    x = _draw(rng, layer.dist_in, (N, layer.C, layer.H, layer.W))
    f = _draw(rng, layer.dist_filt, (layer.K, layer.C, layer.R, layer.S))
    b = None if layer.dist_bias == "none" else _draw(rng, layer.dist_bias, (layer.K,))
    return x, f, b


def make_random_problem(seed, N, C, H, W, K, R, S, dist="u11", with_bias=True):
    """Free-form seeded problem for fuzz / edge-case tests."""
    rng = np.random.default_rng(seed)
    x = _draw(rng, dist, (N, C, H, W))
    f = _draw(rng, dist, (K, C, R, S))
    b = _draw(rng, "u01b", (K,)) if with_bias else None
    return x, f, b


def make_integer_problem(seed, N, C, H, W, K, R, S, lo=-2, hi=2, with_bias=True):
    """Small-integer data: every product and partial sum is an integer below
    2**24, so fp32 arithmetic in any order is exact."""
    rng = np.random.default_rng(seed)
    x = rng.integers(lo, hi + 1, size=(N, C, H, W)).astype(np.float32)
    f = rng.integers(lo, hi + 1, size=(K, C, R, S)).astype(np.float32)
    b = rng.integers(-3, 4, size=(K,)).astype(np.float32) if with_bias else None
    return x, f, b


def make_sgemm_inputs(n, seed=None):
    """(A[n x n] normal(0, 0.01), B[n x n] uniform[0,1)) for the square product of size n."""
    layer = BY_NAME["sgemm_%d" % n]
    x, f, _ = make_layer_inputs(layer, 1, seed)
    return f.reshape(n, n), x.reshape(n, n)


def make_stack_inputs(N, seed=None):
    """Image batch plus (filt, bias) per layer for the five-conv stack."""
    rng = np.random.default_rng(BASE_SEED + 50000 + N if seed is None else seed)
    img = _draw(rng, "u01", (N, CONV1.C, CONV1.H, CONV1.W))
    params = []
    for l in STACK:
        f = _draw(rng, l.dist_filt, (l.K, l.C, l.R, l.S))
        b = _draw(rng, "u01b", (l.K,))
        params.append((f, b))
    return img, params
