"""Seeded synthetic workloads: layer shapes and Gaussian tensors.

This module serves both the GPU path's tests/benchmark and the CPU oracle's
tests, so it deliberately holds none of the method's arithmetic: it only names
layer shapes and draws random numbers.  It imports neither the GPU binding nor
the oracle.

The shapes stand in for the core-convolution shapes of the ImageNet CNNs the
paper measures on (section 7: fp32, 3x3 filters, batch 1, ResNet stage
geometry 56/28/14/7); the values are Gaussian because neither the data set nor
trained weights are needed for a latency or parity measurement.

Recipe: ``numpy.random.default_rng(seed)``; ``standard_normal(float32)`` drawn
in the fixed order x, U_in, core, U_out; weights are then scaled by
fan_in**-0.5 so that every stage keeps unit variance
(fan_in = C for U_in, R1*K*K for core, R2 for U_out).
``seed = 221103715 + 1000*config_id + layer_index``.
"""
from __future__ import annotations

from dataclasses import asdict, dataclass
from typing import Dict, List

import numpy as np

BASE_SEED = 221103715


@dataclass(frozen=True)
class Layer:
    """Shape of one Tucker-2 convolution layer (ranks R1, R2 = the paper's D1, D2)."""
    batch: int
    C: int
    N: int
    H: int
    W: int
    R1: int
    R2: int
    K: int = 3
    stride: int = 1
    pad: int = 1

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad - self.K) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad - self.K) // self.stride + 1

    def asdict(self) -> Dict[str, int]:
        return asdict(self)

    def name(self) -> str:
        return "b%d_c%d_n%d_%dx%d_r%d-%d_k%d_s%d_p%d" % (
            self.batch, self.C, self.N, self.H, self.W, self.R1, self.R2,
            self.K, self.stride, self.pad)


def _round8(v: float) -> int:
    return max(8, int(round(v / 8.0)) * 8)


def config_layers(config_id: int) -> List[Layer]:
    """The five synthetic workloads, numbered 1..5; 6: this library's own throughput set (layers of 4 and a
    14x14 layer at batch sizes that fill the chip); 7: the large-image layers of a VGG-16-shaped network at batch 1."""
    if config_id == 1:   # single layer, the primary parity case
        return [Layer(1, 64, 64, 56, 56, 16, 16)]
    if config_id == 2:   # ResNet-18-shaped sweep, R = C/4
        return [Layer(1, c, c, hw, hw, c // 4, c // 4)
                for c, hw in ((64, 56), (128, 28), (256, 14), (512, 7))]
    if config_id == 3:   # rank sweep at C = N = 256, 14x14
        ranks = (8, 16, 32, 64, 128)
        return [Layer(1, 256, 256, 14, 14, r1, r2) for r1 in ranks for r2 in ranks]
    if config_id == 4:   # stride / batch variants
        out = [Layer(b, 128, 256, 56, 56, 32, 64, 3, 2, 1) for b in (1, 8, 32)]
        out += [Layer(b, 128, 128, 28, 28, 32, 32) for b in (1, 8, 32)]
        return out
    if config_id == 5:   # ResNet-50-style chain of 16 bottleneck 3x3 convs, ranks round(0.3*C) to a multiple of 8
        out: List[Layer] = []
        for c, hw, count in ((64, 56, 3), (128, 28, 4), (256, 14, 6), (512, 7, 3)):
            r = _round8(0.3 * c)
            for i in range(count):
                if i == 0 and c != 64:    # first block of a later stage downsamples
                    out.append(Layer(1, c, c, 2 * hw, 2 * hw, r, r, 3, 2, 1))
                else:
                    out.append(Layer(1, c, c, hw, hw, r, r))
        return out
    if config_id == 6:   # throughput regime: every compute unit gets work
        return [Layer(32, 128, 256, 56, 56, 32, 64, 3, 2, 1), Layer(32, 128, 128, 28, 28, 32, 32),
                Layer(32, 256, 256, 14, 14, 64, 64), Layer(128, 256, 256, 14, 14, 64, 64),
                Layer(128, 128, 128, 28, 28, 32, 32), Layer(64, 128, 256, 56, 56, 32, 64, 3, 2, 1),
                Layer(256, 256, 256, 14, 14, 64, 64), Layer(256, 128, 128, 28, 28, 32, 32)]
    if config_id == 7:   # large images, few channels (section 7.2 names core shapes (64, 32) at 224x224 and 112x112 as its
        # kernel's weak spot); then the deeper VGG-16-shaped layers at a quarter of the channels
        return [Layer(1, 64, 64, 224, 224, 64, 32), Layer(1, 128, 128, 112, 112, 64, 32),
                Layer(1, 128, 256, 56, 56, 32, 64), Layer(1, 256, 256, 56, 56, 64, 64),
                Layer(1, 512, 512, 28, 28, 128, 128), Layer(1, 512, 512, 14, 14, 128, 128)]
    raise ValueError("config_id must be 1..7")


def layer_seed(config_id: int, layer_index: int) -> int:
    return BASE_SEED + 1000 * config_id + layer_index


def make_inputs(layer: Layer, seed: int) -> Dict[str, np.ndarray]:
    """Draw x ~ N(0,1) and weights ~ N(0, 1/fan_in), all float32, C-contiguous."""
    rng = np.random.default_rng(seed)
    L = layer
    x = rng.standard_normal((L.batch, L.C, L.H, L.W), dtype=np.float32)
    U_in = rng.standard_normal((L.C, L.R1), dtype=np.float32)
    core = rng.standard_normal((L.R1, L.R2, L.K, L.K), dtype=np.float32)
    U_out = rng.standard_normal((L.R2, L.N), dtype=np.float32)
    U_in *= np.float32(L.C ** -0.5)
    core *= np.float32((L.R1 * L.K * L.K) ** -0.5)
    U_out *= np.float32(L.R2 ** -0.5)
    return {"x": x, "U_in": U_in, "core": core, "U_out": U_out}


def make_dense_inputs(layer: Layer, seed: int) -> Dict[str, np.ndarray]:
    """Inputs of the undecomposed layer: x ~ N(0,1) and a dense kernel W[C][N][K][K] ~ N(0, 1/(C*K*K))."""
    rng = np.random.default_rng(seed)
    L = layer
    x = rng.standard_normal((L.batch, L.C, L.H, L.W), dtype=np.float32)
    W = rng.standard_normal((L.C, L.N, L.K, L.K), dtype=np.float32)
    W *= np.float32((L.C * L.K * L.K) ** -0.5)
    return {"x": x, "W": W}
