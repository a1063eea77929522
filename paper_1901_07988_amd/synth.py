"""Seeded synthetic inputs shaped like the paper's workloads (Sec. 4: CIFAR ResNet stages at
16/32/64 channels, ImageNet ResNet-152 bottlenecks at 56x56 and 14x14).

This module only draws random numbers and lists layer shapes.  It holds none of the
method's arithmetic, so both the GPU tests and the CPU oracle's tests may use it.
Draw order per layer: x (first layer only), W, gamma, beta; dy last.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional

import numpy as np

DEFAULT_SEED = 190107988


@dataclass(frozen=True)
class LayerShape:
    N: int
    H: int
    W: int
    Cin: int
    Cout: int
    R: int = 3
    S: int = 3
    stride: int = 1
    pad: int = 1

    @property
    def Ho(self):
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Wo(self):
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def M(self):
        return self.N * self.H * self.W

    @property
    def E(self):
        return self.M * self.Cin

    def as_tuple(self):
        return (self.N, self.H, self.W, self.Cin, self.Cout, self.R, self.S, self.stride, self.pad)


@dataclass
class Workload:
    name: str
    shapes: List[LayerShape]
    skip_every: int          # identity skip around each group of this many layers (0: none)
    x_dist: str = "normal"   # "normal" | "relu_normal"
    affine: str = "unit"     # "unit": gamma=1, beta=0 | "random": gamma~U(.5,1.5), beta~N(0,.1)


def he_normal(rng, s: LayerShape):
    std = np.sqrt(2.0 / (s.R * s.S * s.Cin))
    return (rng.standard_normal((s.R, s.S, s.Cin, s.Cout)) * std).astype(np.float32)


def draw_x(rng, s: LayerShape, dist="normal"):
    x = rng.standard_normal((s.N, s.H, s.W, s.Cin)).astype(np.float32)
    if dist == "relu_normal":
        x = np.maximum(x, np.float32(0))
    return x


def draw_affine(rng, C, kind="unit"):
    if kind == "unit":
        return np.ones(C, np.float32), np.zeros(C, np.float32)
    gamma = rng.uniform(0.5, 1.5, C).astype(np.float32)
    beta = (rng.standard_normal(C) * 0.1).astype(np.float32)
    return gamma, beta


def draw_layer(s: LayerShape, seed=DEFAULT_SEED, x_dist="normal", affine="unit"):
    """x, W, gamma, beta, dy for a single layer."""
    rng = np.random.default_rng(seed)
    x = draw_x(rng, s, x_dist)
    w = he_normal(rng, s)
    gamma, beta = draw_affine(rng, s.Cin, affine)
    dy = rng.standard_normal((s.N, s.Ho, s.Wo, s.Cout)).astype(np.float32)
    return x, w, gamma, beta, dy


def draw_stack(wl: Workload, seed=DEFAULT_SEED):
    """x, [(shape, W, gamma, beta)], dy for a stack."""
    rng = np.random.default_rng(seed)
    x = draw_x(rng, wl.shapes[0], wl.x_dist)
    layers = []
    for s in wl.shapes:
        w = he_normal(rng, s)
        gamma, beta = draw_affine(rng, s.Cin, wl.affine)
        layers.append((s, w, gamma, beta))
    last = wl.shapes[-1]
    dy = rng.standard_normal((last.N, last.Ho, last.Wo, last.Cout)).astype(np.float32)
    return x, layers, dy


# ----------------------------------------------------------------------------- the configs
def config1(N=8):
    """Single 3x3 layer, 16 channels at 32x32."""
    return Workload("config1: 3x3 16->16 @32x32 N=%d" % N, [LayerShape(N, 32, 32, 16, 16)], 0)


def config2(N=128, layers=18):
    """CIFAR-ResNet-shaped residual stage: 18 stacked 3x3 layers, 16 channels, 32x32,
    identity skip every 2 layers."""
    return Workload("config2: %dx(3x3 16->16 @32x32) N=%d skip/2" % (layers, N),
                    [LayerShape(N, 32, 32, 16, 16)] * layers, 2)


def config3(N=128, per_stage=18):
    """CIFAR-ResNet wider stages: a stride-2 transition then 3x3 layers at (32ch,16x16), then
    a stride-2 transition and 3x3 layers at (64ch, 8x8).  No skip crosses a transition, so the
    two stages are returned as separate workloads; identity skips every 2 layers where the
    shapes agree (the pair that holds the transition has none)."""
    a = [LayerShape(N, 32, 32, 16, 32, stride=2)] + [LayerShape(N, 16, 16, 32, 32)] * (per_stage - 1)
    b = [LayerShape(N, 16, 16, 32, 64, stride=2)] + [LayerShape(N, 8, 8, 64, 64)] * (per_stage - 1)
    return [Workload("config3a: 16->32 /2 then %dx(3x3 32->32 @16x16) N=%d" % (per_stage - 1, N), a, 2),
            Workload("config3b: 32->64 /2 then %dx(3x3 64->64 @8x8) N=%d" % (per_stage - 1, N), b, 2)]


def config4(N=64, HW=56):
    """ImageNet ResNet-152-style bottleneck at 56x56: 1x1 256->64, 3x3 64->64, 1x1 64->256,
    identity skip around the block."""
    sh = [LayerShape(N, HW, HW, 256, 64, 1, 1, 1, 0), LayerShape(N, HW, HW, 64, 64),
          LayerShape(N, HW, HW, 64, 256, 1, 1, 1, 0)]
    return Workload("config4: bottleneck 256-64-64-256 @%dx%d N=%d" % (HW, HW, N), sh, 3, "relu_normal")


def config5(N=64, blocks=12, HW=14):
    """ImageNet deep-stage bottleneck stack at 14x14: 12 x (1x1 1024->256, 3x3 256->256,
    1x1 256->1024), random per-channel gamma/beta."""
    sh = [LayerShape(N, HW, HW, 1024, 256, 1, 1, 1, 0), LayerShape(N, HW, HW, 256, 256),
          LayerShape(N, HW, HW, 256, 1024, 1, 1, 1, 0)] * blocks
    return Workload("config5: %dx bottleneck 1024-256-256-1024 @%dx%d N=%d" % (blocks, HW, HW, N),
                    sh, 3, "normal", "random")
