"""Seeded synthetic layer shapes and tensors shared by tests, smoke and bench.

Holds no arithmetic of the method: only the five benchmark layer shapes, the paper's
own single-layer shapes (Sec. 5.1-5.3: batch 256, same padding, 14x14x256x256 and
28x28x128x128, kernels 3..11), and the random draws for inputs and weights.
Both the GPU path and the CPU oracle receive the same float32 arrays from here.
"""
from collections import namedtuple

import numpy as np

Layer = namedtuple("Layer", "name N C H W K R S stride pad x_dist")

# The five benchmark layers.  Index 1 is the one the headline metric is quoted on.
CONFIGS = [
    Layer("cfg1_5x5s1_c16k16_32", 1, 16, 32, 32, 16, 5, 5, 1, 2, "uniform"),
    Layer("cfg2_3x3s2_c128k256_56", 32, 128, 56, 56, 256, 3, 3, 2, 1, "uniform"),
    Layer("cfg3_7x7s1_c256k256_28", 32, 256, 28, 28, 256, 7, 7, 1, 3, "relu_normal"),
    Layer("cfg4_7x7s2_c3k64_224", 64, 3, 224, 224, 64, 7, 7, 2, 3, "normal"),
    Layer("cfg5_11x11s4_c3k96_227", 128, 3, 227, 227, 96, 11, 11, 4, 0, "uniform"),
]


def out_hw(L):
    return ((L.H + 2 * L.pad - L.R) // L.stride + 1, (L.W + 2 * L.pad - L.S) // L.stride + 1)


def direct_flops(L):
    OH, OW = out_hw(L)
    return 2.0 * L.N * L.K * L.C * L.R * L.S * OH * OW


def paper_layer(kernel, hw, stride=1, N=256):
    """One of the paper's single-layer shapes: 14x14 maps with 256 channels/filters or
    28x28 with 128, same-padded, standard-normal inputs AND weights."""
    ch = {14: 256, 28: 128}[hw]
    return Layer("paper_%dx%ds%d_%d" % (kernel, kernel, stride, hw), N, ch, hw, hw, ch,
                 kernel, kernel, stride, kernel // 2, "normal_w_normal")


def make_x(L, seed):
    rng = np.random.default_rng(seed)
    shape = (L.N, L.C, L.H, L.W)
    if L.x_dist == "uniform":
        x = rng.uniform(-1.0, 1.0, shape)
    elif L.x_dist == "relu_normal":
        x = np.maximum(rng.standard_normal(shape), 0.0)
    else:
        x = rng.standard_normal(shape)
    return x.astype(np.float32)


def make_w(L, seed):
    rng = np.random.default_rng(seed)
    shape = (L.K, L.C, L.R, L.S)
    std = 1.0 if L.x_dist == "normal_w_normal" else float(np.sqrt(2.0 / (L.C * L.R * L.S)))
    return (rng.standard_normal(shape) * std).astype(np.float32)


def make_layer_tensors(L, index=0):
    """x, w for a layer; seeds 1100+index / 2100+index."""
    return make_x(L, 1100 + index), make_w(L, 2100 + index)
