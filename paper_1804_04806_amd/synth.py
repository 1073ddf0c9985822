"""Seeded synthetic inputs and layer-shape tables for the benchmark workloads.

This module holds no convolution or planner arithmetic: only shapes and random
tensors.  It is the one module that both the HIP-path tests/benchmark and the
CPU-oracle tests draw their inputs from.

Distributions (stand-ins for the paper's ImageNet / CIFAR shaped workloads of
Section 4, which need no dataset to time): activations x ~ U[-1, 1], output
gradients dy ~ U[-1, 1], filters w ~ N(0, 2 / (C*R*S)) (He initialisation),
all float32, drawn from numpy's counter-based Philox generator keyed by
(seed, tensor id) so that any tensor can be regenerated alone.
"""
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Shape:
    """One convolution layer: input (N,C,H,W), K filters of R x S, square stride/pad."""
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    stride: int = 1
    pad: int = 0
    name: str = ""

    @property
    def P(self):
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self):
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def x_shape(self):
        return (self.N, self.C, self.H, self.W)

    @property
    def w_shape(self):
        return (self.K, self.C, self.R, self.S)

    @property
    def y_shape(self):
        return (self.N, self.K, self.P, self.Q)

    @property
    def flops(self):
        """Multiply-adds x 2 of one operation (the same for all three operations)."""
        return 2 * self.N * self.K * self.P * self.Q * self.C * self.R * self.S

    def with_batch(self, n):
        return Shape(n, self.C, self.H, self.W, self.K, self.R, self.S, self.stride, self.pad, self.name)


_X, _W, _DY = 0, 1, 2


def _gen(seed, layer_index, tensor_id):
    return np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF,
                                                     (layer_index << 8) | tensor_id]))


def make_x(s, seed=0, layer_index=0):
    return _gen(seed, layer_index, _X).uniform(-1.0, 1.0, size=s.x_shape).astype(np.float32)


def make_dy(s, seed=0, layer_index=0):
    return _gen(seed, layer_index, _DY).uniform(-1.0, 1.0, size=s.y_shape).astype(np.float32)


def make_w(s, seed=0, layer_index=0):
    std = np.sqrt(2.0 / (s.C * s.R * s.S))
    return (_gen(seed, layer_index, _W).standard_normal(size=s.w_shape) * std).astype(np.float32)


def make_flat(n, kind, seed=0, std=1.0):
    """n values of one of the three distributions as a flat array (pooled benchmark buffers that
    layers of different shapes take views of): kind "x" / "dy" ~ U[-1, 1], "w" ~ N(0, std^2)."""
    g = _gen(seed, 0xFFFF, {"x": _X, "w": _W, "dy": _DY}[kind])
    if kind == "w":
        return (g.standard_normal(size=n) * std).astype(np.float32)
    return g.uniform(-1.0, 1.0, size=n).astype(np.float32)


def to_bf16_bits(a):
    """bfloat16 storage of an fp32 array: round to nearest, ties to even; returns uint16 bits.
    (Input preparation for the bf16 variant: the values the library is handed.)"""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(h):
    """The exact fp32 value of bfloat16 bits."""
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def sample_indices(total, count, seed=0):
    """``count`` distinct flat indices below ``total`` (all of them if total <= count), sorted."""
    if total <= count:
        return np.arange(total, dtype=np.int64)
    g = np.random.Generator(np.random.Philox(key=[seed, 0xABCD]))
    return np.unique(g.integers(0, total, size=count, dtype=np.int64))


# ---- workload tables -------------------------------------------------------------

MIB = 1 << 20


def config_small():
    """One small layer whose 64 KiB limit no workspace algorithm fits."""
    return [Shape(8, 16, 16, 16, 32, 3, 3, 1, 1, "small3x3")]


def config_alexnet(batch=256):
    """AlexNet-shaped (single-column, ungrouped) five-layer convolution stack."""
    return [
        Shape(batch, 3, 227, 227, 96, 11, 11, 4, 0, "conv1"),
        Shape(batch, 96, 27, 27, 256, 5, 5, 1, 2, "conv2"),
        Shape(batch, 256, 13, 13, 384, 3, 3, 1, 1, "conv3"),
        Shape(batch, 384, 13, 13, 384, 3, 3, 1, 1, "conv4"),
        Shape(batch, 384, 13, 13, 256, 3, 3, 1, 1, "conv5"),
    ]


def config_resnet18(batch=256):
    """ResNet-18-shaped convolution layers in network order (20 layers, 11 unique)."""
    out = [Shape(batch, 3, 224, 224, 64, 7, 7, 2, 3, "stem")]
    out += [Shape(batch, 64, 56, 56, 64, 3, 3, 1, 1, f"s1.conv{i}") for i in range(4)]
    c, h = 64, 56
    for stage, k in ((2, 128), (3, 256), (4, 512)):
        out.append(Shape(batch, c, h, h, k, 3, 3, 2, 1, f"s{stage}.down3x3"))
        out.append(Shape(batch, c, h, h, k, 1, 1, 2, 0, f"s{stage}.proj1x1"))
        h //= 2
        out += [Shape(batch, k, h, h, k, 3, 3, 1, 1, f"s{stage}.conv{i}") for i in range(3)]
        c = k
    return out


def config_densenet_block(batch=64):
    """DenseNet-BC-style block at 32 x 32: twelve (1x1 -> 128, 3x3 128 -> 32) pairs."""
    out = []
    for i in range(12):
        out.append(Shape(batch, 64 + 32 * i, 32, 32, 128, 1, 1, 1, 0, f"l{i}.1x1"))
        out.append(Shape(batch, 128, 32, 32, 32, 3, 3, 1, 1, f"l{i}.3x3"))
    return out


def config_resnet50(batch=256):
    """ResNet-50-shaped layers, stride on the 3x3 of the first block of a stage (53 layers)."""
    out = [Shape(batch, 3, 224, 224, 64, 7, 7, 2, 3, "stem")]
    c, h = 64, 56
    for stage, (mid, count) in enumerate(((64, 3), (128, 4), (256, 6), (512, 3)), start=1):
        wide = 4 * mid
        for blk in range(count):
            s = 2 if (blk == 0 and stage > 1) else 1
            out.append(Shape(batch, c, h, h, mid, 1, 1, 1, 0, f"s{stage}b{blk}.reduce"))
            out.append(Shape(batch, mid, h, h, mid, 3, 3, s, 1, f"s{stage}b{blk}.conv3x3"))
            ho = h // s
            out.append(Shape(batch, mid, ho, ho, wide, 1, 1, 1, 0, f"s{stage}b{blk}.expand"))
            if blk == 0:
                out.append(Shape(batch, c, h, h, wide, 1, 1, s, 0, f"s{stage}b{blk}.proj"))
            c, h = wide, ho
    return out
