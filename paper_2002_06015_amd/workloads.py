"""Seeded synthetic workloads: layer shapes and input tensors only.

This module holds none of the method's arithmetic.  It serves both the GPU
library's tests/benchmark and the CPU oracle's tests with the *same* host
arrays.  Shapes are those of ResNet-50 (the network the paper trains, Sec. 7);
values are synthetic stand-ins for ImageNet activations and gradients:

    activations   a = max(0, z),  z ~ N(0, 1)          ("post-ReLU")
    output grads  g ~ N(0, (1e-3)^2)                    (per-sample d log p / d s)
    weight grads  dW ~ N(0, (1e-3)^2), shape [dG, dA]
    BN grads      g_gamma, g_beta ~ N(0, (1e-3)^2), shape [N, C]

all float32 from ``numpy.random.default_rng(seed)``.
"""
from __future__ import annotations

from typing import Dict, List, NamedTuple, Tuple

import numpy as np

GAMMA = 1e-3          # factor-level damping sqrt(lambda)
DECAY = 0.95          # running-average decay
BN_LAMBDA = 1e-6      # BatchNorm damping lambda = GAMMA**2
GRAD_SIGMA = 1e-3


class Layer(NamedTuple):
    """One K-FAC layer. A fully-connected layer is k=1, stride=1, pad=0, h_in=w_in=1."""
    N: int
    c_in: int
    c_out: int
    k: int
    stride: int
    pad: int
    h_in: int
    w_in: int
    bias: int

    @property
    def h(self) -> int:
        return (self.h_in + 2 * self.pad - self.k) // self.stride + 1

    @property
    def w(self) -> int:
        return (self.w_in + 2 * self.pad - self.k) // self.stride + 1

    @property
    def dA(self) -> int:
        return self.c_in * self.k * self.k + (1 if self.bias else 0)

    @property
    def dG(self) -> int:
        return self.c_out

    @property
    def M(self) -> int:
        return self.N * self.h * self.w


def fc_layer(N: int, d_in: int, d_out: int, bias: int = 1) -> Layer:
    return Layer(N, d_in, d_out, 1, 1, 0, 1, 1, bias)


def conv_layer(N: int, c_in: int, c_out: int, k: int, stride: int, pad: int, h_in: int,
               bias: int = 1) -> Layer:
    return Layer(N, c_in, c_out, k, stride, pad, h_in, h_in, bias)


def resnet50_layers(N: int, variant: str = "v1", bias: int = 1) -> Tuple[List[Layer], List[Tuple[int, int]]]:
    """The 54 K-FAC layers (53 conv + 1 FC) of ResNet-50 at 224x224 input, in forward
    order, and the 53 BatchNorm layers as (C, h) pairs (one after every conv).

    v1 puts the stride of stages 3-5 on the first 1x1 of the first bottleneck;
    v1.5 puts it on the 3x3.  The downsample 1x1 carries the stride in both.
    """
    if variant not in ("v1", "v1.5"):
        raise ValueError("variant must be 'v1' or 'v1.5'")
    layers: List[Layer] = [conv_layer(N, 3, 64, 7, 2, 3, 224, bias)]
    res = 56                      # after the parameter-free 3x3/2 max-pool
    c_prev = 64
    for stage, (blocks, mid) in enumerate(zip([3, 4, 6, 3], [64, 128, 256, 512])):
        out = 4 * mid
        for b in range(blocks):
            stride = 2 if (b == 0 and stage > 0) else 1
            s1, s3 = (stride, 1) if variant == "v1" else (1, stride)
            r_in = res
            r_mid = (r_in - 1) // s1 + 1
            layers.append(conv_layer(N, c_prev, mid, 1, s1, 0, r_in, bias))
            layers.append(conv_layer(N, mid, mid, 3, s3, 1, r_mid, bias))
            r_out = (r_mid + 2 - 3) // s3 + 1
            layers.append(conv_layer(N, mid, out, 1, 1, 0, r_out, bias))
            if b == 0:
                layers.append(conv_layer(N, c_prev, out, 1, stride, 0, r_in, bias))
            c_prev, res = out, r_out
    layers.append(fc_layer(N, 2048, 1000, bias))
    bns = [(L.c_out, L.h) for L in layers[:-1]]
    return layers, bns


def flops(layer: Layer) -> Dict[str, float]:
    """Algorithmic flop counts of one step for one layer: symmetric Gram matrices
    M*d*(d+1), SPD inverses n^3, preconditioning 2 dG^2 dA + 2 dG dA^2."""
    dA, dG, M = layer.dA, layer.dG, layer.M
    return {
        "stats_A": float(M) * dA * (dA + 1),
        "stats_G": float(M) * dG * (dG + 1),
        "inv": float(dA) ** 3 + float(dG) ** 3,
        "precond": 2.0 * dG * dG * dA + 2.0 * dG * dA * dA,
    }


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest-even bfloat16, returned as float32 holding the rounded value."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(np.shape(x))


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """The uint16 bit patterns of values that are already bf16-representable."""
    return (np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16).reshape(np.shape(x))


def make_act(layer: Layer, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    shape = (layer.N, layer.c_in, layer.h_in, layer.w_in)
    a = rng.standard_normal(shape, dtype=np.float32)
    np.maximum(a, 0.0, out=a)
    return a


def make_grad_out(layer: Layer, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed + 7_000_000)
    g = rng.standard_normal((layer.N, layer.c_out, layer.h, layer.w), dtype=np.float32)
    g *= np.float32(GRAD_SIGMA)
    return g


def make_grad_W(layer: Layer, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed + 13_000_000)
    g = rng.standard_normal((layer.dG, layer.dA), dtype=np.float32)
    g *= np.float32(GRAD_SIGMA)
    return g


def make_bn_grads(N: int, C: int, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    rng = np.random.default_rng(seed + 19_000_000)
    gg = rng.standard_normal((N, C), dtype=np.float32) * np.float32(GRAD_SIGMA)
    gb = rng.standard_normal((N, C), dtype=np.float32) * np.float32(GRAD_SIGMA)
    return gg, gb


def make_bn_nchw(N: int, C: int, HW: int, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """(dy, xhat): output gradient ~ N(0,(1e-3)^2) and normalised input ~ N(0,1), [N, C, HW]."""
    rng = np.random.default_rng(seed + 23_000_000)
    dy = rng.standard_normal((N, C, HW), dtype=np.float32) * np.float32(GRAD_SIGMA)
    xhat = rng.standard_normal((N, C, HW), dtype=np.float32)
    return dy, xhat


def layer_seed(config: int, layer_index: int, second_batch: bool = False) -> int:
    return 1000 * config + layer_index + (500 if second_batch else 0)


def stale_subset(n_layers: int, seed: int, fraction: float = 0.25) -> np.ndarray:
    """Indices of the layers whose inverses are refreshed in the stale-statistics
    configuration: a seeded random ceil(fraction*n) subset."""
    m = int(np.ceil(fraction * n_layers))
    return np.sort(np.random.default_rng(seed).permutation(n_layers)[:m])


def config_layers(config: int) -> List[Layer]:
    """Layer lists of the benchmark configurations 1-5."""
    if config == 1:
        return [fc_layer(32, 64, 32)]
    if config == 2:
        return [conv_layer(32, 64, 64, 3, 1, 1, 56)]
    if config == 3:
        return [conv_layer(32, 512, 512, 3, 1, 1, 7), fc_layer(32, 2048, 1000)]
    if config == 4:
        return resnet50_layers(32)[0]
    if config == 5:
        return resnet50_layers(128)[0]
    raise ValueError("config must be 1..5")
