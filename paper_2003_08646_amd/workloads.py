"""Seeded synthetic layers shaped like the paper's workloads (Sec. 4: SVHN / CIFAR nets,
a ResNet-18 variant, VGG-style stacks).  The datasets and trained weights themselves are not
used; only their layer shapes and value distributions are imitated:

* activations: post-ReLU-like, ``max(N(0,1), 0)`` (or ``U(0,1)`` for the smallest case; the
  first VGG layer sees a normalised image, ``N(0,1)``);
* filters: He-normal, ``N(0, 2/(9*C))``.

This module only draws random numbers and names shapes.  It contains none of the method's
arithmetic and is the one module shared by the oracle-side tests and the GPU side.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Layer:
    name: str
    N: int
    C: int
    K: int
    H: int
    W: int
    pad: int = 1
    m: int = 2
    bits: int = 8
    seed: int = 0
    x_dist: str = "relu_normal"  # relu_normal | uniform01 | normal
    bits_w: int | None = None    # width of the filter codes when it differs from bits

    @property
    def Ho(self) -> int:
        return self.H + 2 * self.pad - 2

    @property
    def Wo(self) -> int:
        return self.W + 2 * self.pad - 2

    @property
    def direct_ops(self) -> int:
        """Multiply-adds x2 of the direct 3x3 convolution (Eq. 1)."""
        return 2 * self.N * self.K * self.C * self.Ho * self.Wo * 9

    def with_(self, **kw) -> "Layer":
        d = dict(self.__dict__)
        d.update(kw)
        return Layer(**d)


def make_inputs(layer: Layer):
    """(X NCHW fp32, W KCRS fp32), a pure function of the layer's shape, distribution, seed."""
    rng = np.random.default_rng(layer.seed)
    shape = (layer.N, layer.C, layer.H, layer.W)
    if layer.x_dist == "uniform01":
        X = rng.random(shape, dtype=np.float32)
    elif layer.x_dist == "normal":
        X = rng.standard_normal(shape, dtype=np.float32)
    elif layer.x_dist == "relu_normal":
        X = np.maximum(rng.standard_normal(shape, dtype=np.float32), np.float32(0))
    else:
        raise ValueError(layer.x_dist)
    std = np.float32(np.sqrt(2.0 / (9.0 * layer.C)))
    Wt = rng.standard_normal((layer.K, layer.C, 3, 3), dtype=np.float32) * std
    return np.ascontiguousarray(X), np.ascontiguousarray(Wt)


# The five benchmark configurations.
CFG1 = Layer("cfg1_n1_c16_k16_32", 1, 16, 16, 32, 32, seed=0, x_dist="uniform01")
CFG2 = Layer("cfg2_n128_c64_k64_32", 128, 64, 64, 32, 32, seed=2)
CFG3_M2 = Layer("cfg3_n64_c128_k128_56_m2", 64, 128, 128, 56, 56, m=2, seed=3)
CFG3_M4 = Layer("cfg3_n64_c128_k128_56_m4", 64, 128, 128, 56, 56, m=4, seed=3)
CFG4 = Layer("cfg4_n64_c512_k512_14", 64, 512, 512, 14, 14, seed=4)
# Not a paper workload: a layer wide enough (16 GEMMs of 2048 x 4096 x 2048) that the product
# kernel is bound by the matrix units rather than by memory; shows its quality on its own.
PROBE = Layer("probe_n16_c2048_k2048_32", 16, 2048, 2048, 32, 32, seed=9)

_VGG_PLAN = [(3, 64, 224), (64, 64, 224), (64, 128, 112), (128, 128, 112), (128, 256, 56),
             (256, 256, 56), (256, 256, 56), (256, 512, 28), (512, 512, 28), (512, 512, 28),
             (512, 512, 14), (512, 512, 14), (512, 512, 14)]


def vgg16_layers(batch: int = 16):
    """The thirteen 3x3 layers of a VGG-16-shaped network at 224x224, independent inputs."""
    out = []
    for i, (c, k, hw) in enumerate(_VGG_PLAN):
        out.append(Layer(f"vgg16_conv{i + 1}_c{c}_k{k}_{hw}", batch, c, k, hw, hw,
                         seed=500 + i + 1, x_dist="normal" if i == 0 else "relu_normal"))
    return out


CONFIGS = {
    "cfg1": [CFG1],
    "cfg2": [CFG2],
    "cfg3": [CFG3_M2, CFG3_M4],
    "cfg4": [CFG4],
    "cfg5": vgg16_layers(),
}
