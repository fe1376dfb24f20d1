"""Seeded synthetic convolution layers shaped like the paper's CNN benchmarks.

The paper's throughput table (Section 6.3, Table 1) trains AlexNet, VGG-19,
ResNet-50 and MobileNet in 32-bit floats but names no dataset, batch size or
layer list, so the layers below are synthetic stand-ins of those networks'
well-known convolution shapes.  This module only draws random inputs and packs
them as fp32 or bf16; it contains none of the convolution arithmetic and is
the one module the HIP path's callers and the CPU oracle's callers share.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np


@dataclass(frozen=True)
class Layer:
    name: str
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    stride: int
    pad: int
    groups: int
    seed: int
    x_dist: str = "normal"   # "normal" -> N(0,1); "uniform" -> U[-1,1]
    note: str = ""
    stride_w: int = -1       # -1: same as stride (which then is the vertical stride)
    pad_w: int = -1          # -1: same as pad

    @property
    def strides(self) -> Tuple[int, int]:
        return (self.stride, self.stride if self.stride_w < 0 else self.stride_w)

    @property
    def pads(self) -> Tuple[int, int]:
        return (self.pad, self.pad if self.pad_w < 0 else self.pad_w)

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pads[0] - self.R) // self.strides[0] + 1

    @property
    def Q(self) -> int:
        return (self.W + 2 * self.pads[1] - self.S) // self.strides[1] + 1

    @property
    def x_shape(self) -> Tuple[int, int, int, int]:
        return (self.N, self.C, self.H, self.W)

    @property
    def w_shape(self) -> Tuple[int, int, int, int]:
        return (self.K, self.C // self.groups, self.R, self.S)

    @property
    def y_shape(self) -> Tuple[int, int, int, int]:
        return (self.N, self.K, self.P, self.Q)

    @property
    def flops(self) -> int:
        """Nominal FLOPs of one pass (the same count is used for all three)."""
        return 2 * self.N * self.K * self.P * self.Q * (self.C // self.groups) * self.R * self.S

    def conv_args(self):
        """(N,C,H,W,K,R,S,stride_h,stride_w,pad_h,pad_w,groups)"""
        return (self.N, self.C, self.H, self.W, self.K, self.R, self.S,
                self.strides[0], self.strides[1], self.pads[0], self.pads[1], self.groups)


# seed = 16 * (index of the configuration group) + (index of the layer in it)
LAYERS: Dict[str, Layer] = {l.name: l for l in [
    Layer("1", 2, 3, 16, 16, 8, 3, 3, 1, 1, 1, seed=0, note="tiny 3x3"),
    Layer("2a", 64, 256, 14, 14, 256, 3, 3, 1, 1, 1, seed=16, note="ResNet-50 bottleneck 3x3"),
    Layer("2b", 64, 1024, 14, 14, 256, 1, 1, 1, 0, 1, seed=17, note="ResNet-50 bottleneck 1x1"),
    Layer("2c", 64, 128, 28, 28, 128, 3, 3, 2, 1, 1, seed=18, note="ResNet-50 3x3 stride 2"),
    Layer("3", 128, 3, 224, 224, 64, 11, 11, 4, 2, 1, seed=32, x_dist="uniform",
          note="AlexNet first layer"),
    Layer("4a", 64, 64, 224, 224, 64, 3, 3, 1, 1, 1, seed=48, note="VGG 3x3 at 224x224"),
    Layer("4b", 64, 512, 28, 28, 512, 3, 3, 1, 1, 1, seed=49, note="VGG 3x3 at 28x28"),
    Layer("5a", 128, 512, 14, 14, 512, 3, 3, 1, 1, 512, seed=64, note="MobileNet depthwise 3x3"),
    Layer("5b", 128, 512, 14, 14, 512, 1, 1, 1, 0, 1, seed=65, note="MobileNet pointwise 1x1"),
]}


def custom_layer(name, N, C, H, W, K, R, S, stride=1, pad=0, groups=1, seed=1234, x_dist="normal"):
    """stride and pad may be ints or (vertical, horizontal) pairs."""
    sh, sw = (stride, -1) if isinstance(stride, int) else stride
    ph, pw = (pad, -1) if isinstance(pad, int) else pad
    return Layer(name, N, C, H, W, K, R, S, sh, ph, groups, seed, x_dist, "", sw, pw)


def make_inputs(layer: Layer):
    """Draw (x, w, dy) as float32, in that order, from PCG64(layer.seed).

    x ~ N(0,1) (or U[-1,1]); w ~ N(0, 2/fan_in) with fan_in = (C/groups)*R*S
    (Kaiming-normal, no truncation); dy ~ N(0,1).
    """
    rng = np.random.Generator(np.random.PCG64(layer.seed))
    if layer.x_dist == "uniform":
        x = rng.uniform(-1.0, 1.0, size=layer.x_shape).astype(np.float32)
    else:
        x = rng.standard_normal(size=layer.x_shape, dtype=np.float32)
    fan_in = (layer.C // layer.groups) * layer.R * layer.S
    w = rng.standard_normal(size=layer.w_shape, dtype=np.float32)
    w *= np.float32(np.sqrt(2.0 / fan_in))
    dy = rng.standard_normal(size=layer.y_shape, dtype=np.float32)
    return x, w, dy


def make_epilogue_inputs(layer: Layer):
    """Inputs of the fused epilogues, drawn from PCG64(layer.seed + 1000): bias ~ N(0,1) per output channel
    (float32) and act = max(0, z), z ~ N(0,1), shaped like x: the output of a rectified linear unit, about half of it
    exactly zero."""
    rng = np.random.Generator(np.random.PCG64(layer.seed + 1000))
    bias = rng.standard_normal(size=(layer.K,), dtype=np.float32)
    act = np.maximum(rng.standard_normal(size=layer.x_shape, dtype=np.float32), np.float32(0.0))
    return bias, act


def make_bn_inputs(N, C, H, W, seed):
    """Inputs of the batch-normalisation passes, float32, drawn from PCG64(seed) in the order x, dy, gamma, beta.
    x is shaped like the output of a convolution layer in training: per channel a mean offset m_c ~ N(0, 1) and a
    scale s_c ~ U[0.5, 2], x = m_c + s_c * N(0, 1); dy ~ N(0, 1); gamma ~ N(1, 0.25); beta ~ N(0, 1)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal(size=(N, C, H, W), dtype=np.float32)
    m = rng.standard_normal(size=(1, C, 1, 1), dtype=np.float32)
    s = rng.uniform(0.5, 2.0, size=(1, C, 1, 1)).astype(np.float32)
    x = (m + s * x).astype(np.float32)
    dy = rng.standard_normal(size=(N, C, H, W), dtype=np.float32)
    gamma = (1.0 + 0.5 * rng.standard_normal(size=(C,), dtype=np.float32)).astype(np.float32)
    beta = rng.standard_normal(size=(C,), dtype=np.float32)
    return x, dy, gamma, beta


# Batch-normalisation shapes of the benchmark: the tensor behind the ResNet-50 3x3 bottleneck layer and the one
# behind its first (7x7 stride-2) layer.  (name, N, C, H, W)
BN_SHAPES = [("bn14", 64, 256, 14, 14), ("bn112", 64, 64, 112, 112)]


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns.
    NaN inputs are not expected in the synthetic data and are not special-cased."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def sample_indices(shape, count, seed):
    """A seeded sample of flat indices into a 4-d tensor that always includes
    the four spatial corners, points on each edge and interior points of the
    first and last (dim0, dim1) planes, followed by uniform random picks."""
    d0, d1, d2, d3 = shape
    total = d0 * d1 * d2 * d3
    rng = np.random.Generator(np.random.PCG64(seed))
    forced = []
    for a in sorted({0, d0 - 1}):
        for b in sorted({0, d1 - 1}):
            for i in sorted({0, d2 // 2, d2 - 1}):
                for j in sorted({0, d3 // 2, d3 - 1}):
                    forced.append(((a * d1 + b) * d2 + i) * d3 + j)
    forced = np.asarray(forced, dtype=np.int64)
    if count >= total:
        return np.arange(total, dtype=np.int64)
    extra = rng.integers(0, total, size=max(0, count - forced.size), dtype=np.int64)
    return np.unique(np.concatenate([forced, extra]))


# Further layer shapes of the networks the benchmark layers come from (ResNet-50, VGG, MobileNet): a second
# sweep for `bench.py --sweep`; not part of the nine benchmark layers.  (name, N, C, H, W, K, R, stride, pad, groups)
MORE_SHAPES = [
    ("resnet stem 7x7 s2 3->64 224", 64, 3, 224, 224, 64, 7, 2, 3, 1),
    ("resnet 3x3 64 56x56", 64, 64, 56, 56, 64, 3, 1, 1, 1),
    ("resnet 1x1 64->256 56x56", 64, 64, 56, 56, 256, 1, 1, 0, 1),
    ("resnet 1x1 256->64 56x56", 64, 256, 56, 56, 64, 1, 1, 0, 1),
    ("resnet 1x1 s2 256->512 56->28", 64, 256, 56, 56, 512, 1, 2, 0, 1),
    ("resnet 3x3 128 28x28", 64, 128, 28, 28, 128, 3, 1, 1, 1),
    ("resnet 1x1 512->128 28x28", 64, 512, 28, 28, 128, 1, 1, 0, 1),
    ("resnet 3x3 s2 256 28->14", 64, 256, 28, 28, 256, 3, 2, 1, 1),
    ("resnet 3x3 512 7x7", 64, 512, 7, 7, 512, 3, 1, 1, 1),
    ("resnet 1x1 512->2048 7x7", 64, 512, 7, 7, 2048, 1, 1, 0, 1),
    ("resnet 1x1 2048->512 7x7", 64, 2048, 7, 7, 512, 1, 1, 0, 1),
    ("vgg 3x3 64->128 112x112", 32, 64, 112, 112, 128, 3, 1, 1, 1),
    ("vgg 3x3 256 56x56", 32, 256, 56, 56, 256, 3, 1, 1, 1),
    ("vgg 3x3 512 14x14", 64, 512, 14, 14, 512, 3, 1, 1, 1),
    ("mobilenet dw 32 112x112", 128, 32, 112, 112, 32, 3, 1, 1, 32),
    ("mobilenet dw s2 64 112->56", 128, 64, 112, 112, 64, 3, 2, 1, 64),
    ("mobilenet dw 128 56x56", 128, 128, 56, 56, 128, 3, 1, 1, 128),
    ("mobilenet dw s2 128 56->28", 128, 128, 56, 56, 128, 3, 2, 1, 128),
    ("mobilenet dw 256 28x28", 128, 256, 28, 28, 256, 3, 1, 1, 256),
    ("mobilenet dw s2 256 28->14", 128, 256, 28, 28, 256, 3, 2, 1, 256),
    ("mobilenet dw s2 512 14->7", 128, 512, 14, 14, 512, 3, 2, 1, 512),
    ("mobilenet dw 1024 7x7", 128, 1024, 7, 7, 1024, 3, 1, 1, 1024),
    ("mobilenet pw 32->64 112x112", 128, 32, 112, 112, 64, 1, 1, 0, 1),
    ("mobilenet pw 1024->1024 7x7", 128, 1024, 7, 7, 1024, 1, 1, 0, 1),
]
