"""Seeded synthetic inputs and the layer shapes the benchmarks and tests run on.

This module holds no arithmetic of the convolution itself: it only names layer
shapes and fills arrays from a counter-based generator, so that the CPU oracle
and the HIP path can be fed bit-identical inputs without sharing any code of
the method.

The shapes stand in for the AlexNet / VGG-16 / GoogLeNet layers the paper timed
(section IV): the paper needs only the layer shapes (single image, stride 1),
not trained weights or images, so inputs are drawn i.i.d. from the stated
distributions.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

_MASK64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_MIX1 = np.uint64(0xBF58476D1CE4E5B9)
_MIX2 = np.uint64(0x94D049BB133111EB)


def splitmix64(seed: int, index: np.ndarray) -> np.ndarray:
    """Counter-based 64-bit hash: element `index` of the stream `seed`.

    The finaliser of the SplitMix64 generator applied to seed + (index+1)*gamma;
    every element is independent of the others, so any slice of a stream can be
    generated on its own.
    """
    with np.errstate(over="ignore"):
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + (index.astype(np.uint64) + np.uint64(1)) * _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _MIX1
        z = (z ^ (z >> np.uint64(27))) * _MIX2
        z = z ^ (z >> np.uint64(31))
    return z


def _unit24(seed: int, index: np.ndarray) -> np.ndarray:
    """Top 24 bits of the hash as an integer in [0, 2^24)."""
    return (splitmix64(seed, index) >> np.uint64(40)).astype(np.float64)


def uniform(seed: int, count: int, lo: float, hi: float) -> np.ndarray:
    """`count` float32 values uniform on [lo, hi) (24-bit resolution)."""
    idx = np.arange(count, dtype=np.uint64)
    u = _unit24(seed, idx) / float(1 << 24)
    return (lo + (hi - lo) * u).astype(np.float32)


def normal(seed: int, count: int, std: float) -> np.ndarray:
    """`count` float32 values from N(0, std^2): Box-Muller on two hashed uniforms per value."""
    idx = np.arange(count, dtype=np.uint64)
    u1 = (_unit24(seed, idx * np.uint64(2)) + 1.0) / float(1 << 24)          # (0, 1]
    u2 = _unit24(seed, idx * np.uint64(2) + np.uint64(1)) / float(1 << 24)    # [0, 1)
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)
    return (std * z).astype(np.float32)


def small_integers(seed: int, count: int, lo: int, hi: int) -> np.ndarray:
    """`count` float32 values that are integers uniform on [lo, hi] (inclusive)."""
    idx = np.arange(count, dtype=np.uint64)
    span = np.uint64(hi - lo + 1)
    v = (splitmix64(seed, idx) >> np.uint64(33)) % span
    return (v.astype(np.int64) + lo).astype(np.float32)


@dataclasses.dataclass(frozen=True)
class Layer:
    """One multi-channel multi-kernel convolution problem (zero padding; stride 1 unless stated)."""
    name: str
    n: int
    c: int
    h: int
    w: int
    m: int
    k: int
    pad: int
    input_dist: str = "u01"      # "u01": uniform[0,1) (post-ReLU-like); "u11": uniform[-1,1)
    kernel_dist: str = "he"      # "he": N(0, sqrt(2/(C k^2))); "u11": uniform[-1,1)
    seed: int = 0
    stride: int = 1

    @property
    def q(self) -> int:          # output height
        return (self.h + 2 * self.pad - self.k) // self.stride + 1

    @property
    def p(self) -> int:          # output width
        return (self.w + 2 * self.pad - self.k) // self.stride + 1

    @property
    def flops(self) -> int:
        return 2 * self.n * self.m * self.c * self.k * self.k * self.q * self.p

    def input_shape(self):
        return (self.n, self.c, self.h, self.w)

    def kernel_shape(self):
        return (self.m, self.c, self.k, self.k)

    def output_shape(self):
        return (self.n, self.m, self.q, self.p)


_SEED_BASE = 0x170404428

# The five benchmark configurations (the fifth is a sweep of three shapes).
LAYERS = {
    "cfg1_tiny": Layer("cfg1_tiny", 1, 16, 32, 32, 16, 3, 1, "u11", "u11", _SEED_BASE + 16 * 1),
    "cfg2_googlenet5x5": Layer("cfg2_googlenet5x5", 1, 32, 28, 28, 96, 5, 2, "u01", "he", _SEED_BASE + 16 * 2),
    "cfg3_alexnet_conv2": Layer("cfg3_alexnet_conv2", 1, 96, 27, 27, 256, 5, 2, "u01", "he", _SEED_BASE + 16 * 3),
    "cfg4_vgg_early": Layer("cfg4_vgg_early", 1, 64, 224, 224, 64, 3, 1, "u01", "he", _SEED_BASE + 16 * 4),
    "cfg5a_vgg_deep56": Layer("cfg5a_vgg_deep56", 8, 256, 56, 56, 256, 3, 1, "u01", "he", _SEED_BASE + 16 * 5),
    "cfg5b_vgg_deep28": Layer("cfg5b_vgg_deep28", 8, 512, 28, 28, 512, 3, 1, "u01", "he", _SEED_BASE + 16 * 6),
    "cfg5c_vgg_deep14": Layer("cfg5c_vgg_deep14", 8, 512, 14, 14, 512, 3, 1, "u01", "he", _SEED_BASE + 16 * 7),
}

# The deep VGG-like shape varied along the axes the paper leaves out (stride, even kernel side) and
# reduced to the 1 x 1 building block of section III-A; measured beside the benchmark layers.
GENERALISED_LAYERS = {
    "gen_vgg56_stride2": Layer("gen_vgg56_stride2", 8, 256, 56, 56, 256, 3, 1, "u01", "he", _SEED_BASE + 16 * 8, 2),
    "gen_vgg56_k4": Layer("gen_vgg56_k4", 8, 256, 56, 56, 256, 4, 2, "u01", "he", _SEED_BASE + 16 * 9),
    "gen_vgg56_1x1": Layer("gen_vgg56_1x1", 8, 256, 56, 56, 256, 1, 0, "u01", "he", _SEED_BASE + 16 * 10),
    # three-channel first layers of the networks the paper takes its layers from: 3 x 3 (VGG) and 7 x 7 with stride 2
    "gen_rgb224_k3": Layer("gen_rgb224_k3", 8, 3, 224, 224, 64, 3, 1, "u01", "he", _SEED_BASE + 16 * 11),
    "gen_rgb224_k7_stride2": Layer("gen_rgb224_k7_stride2", 8, 3, 224, 224, 64, 7, 3, "u01", "he", _SEED_BASE + 16 * 12, 2),
}


def make_input(layer: Layer) -> np.ndarray:
    """Input tensor I[N][C][H][W], float32, from the layer's seed."""
    count = layer.n * layer.c * layer.h * layer.w
    if layer.input_dist == "u01":
        flat = uniform(layer.seed, count, 0.0, 1.0)
    elif layer.input_dist == "u11":
        flat = uniform(layer.seed, count, -1.0, 1.0)
    elif layer.input_dist == "int":
        flat = small_integers(layer.seed, count, 0, 8)
    else:
        raise ValueError(f"unknown input distribution {layer.input_dist!r}")
    return flat.reshape(layer.input_shape())


def make_kernel(layer: Layer) -> np.ndarray:
    """Kernel tensor K[M][C][k][k], float32, from the layer's seed + 1."""
    count = layer.m * layer.c * layer.k * layer.k
    seed = layer.seed + 1
    if layer.kernel_dist == "he":
        flat = normal(seed, count, math.sqrt(2.0 / (layer.c * layer.k * layer.k)))
    elif layer.kernel_dist == "u11":
        flat = uniform(seed, count, -1.0, 1.0)
    elif layer.kernel_dist == "int":
        flat = small_integers(seed, count, -4, 4)
    else:
        raise ValueError(f"unknown kernel distribution {layer.kernel_dist!r}")
    return flat.reshape(layer.kernel_shape())


def sample_points(layer: Layer, count: int, seed: int = 7) -> np.ndarray:
    """`count` output coordinates (n, m, q, p), int32, spread over the whole output and
    always including the four corners of the first and last plane."""
    idx = np.arange(count, dtype=np.uint64)
    hsh = splitmix64(layer.seed + 1000 + seed, idx)
    total = layer.n * layer.m * layer.q * layer.p
    flat = (hsh % np.uint64(total)).astype(np.int64)
    pts = np.stack(np.unravel_index(flat, layer.output_shape()), axis=1).astype(np.int32)
    corners = []
    for (n, m) in ((0, 0), (layer.n - 1, layer.m - 1)):
        for q in (0, layer.q - 1):
            for p in (0, layer.p - 1):
                corners.append((n, m, q, p))
    pts[: min(len(corners), count)] = np.array(corners, dtype=np.int32)[: min(len(corners), count)]
    return pts
