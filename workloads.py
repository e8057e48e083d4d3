"""Seeded synthetic inputs and the layer tables of the benchmark configurations.

This module holds NO convolution arithmetic: it only produces input tensors
(X, W, G) and names shapes.  It is the single piece shared by the CPU oracle's
tests and the GPU path's tests/bench, so both sides see identical bits.

Inputs stand in for CIFAR-10 batches and for the layers of the paper's
networks (Sec. IV, Table I: 32x32x3 images, float32, [N,H,W,C]); conv results
depend on shapes and value scale only, so nothing of the dataset is needed.

Generator: a counter-based splitmix64 stream per tensor.  Element i of a
tensor with stream key k is a pure function of (k, i), so any sub-range can be
regenerated independently.
  uniform[-1,1)  : (u >> 40) * 2^-23 - 1          (24 random bits, exact in fp32)
  N(0,1)         : Box-Muller on two 53-bit uniforms, in fp64, rounded to fp32
  Kaiming-normal : N(0,1) * sqrt(2 / (FH*FW*IC))
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 20230508
_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix64(z: np.ndarray) -> np.ndarray:
    """The splitmix64 output function applied to an array of uint64 states."""
    with np.errstate(over="ignore"):
        z = (z + np.uint64(0x9E3779B97F4A7C15)) & _M64
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
        return z ^ (z >> np.uint64(31))


def stream_key(*parts) -> int:
    """Mix integers/strings into one 64-bit stream key (order-sensitive)."""
    k = np.array([BASE_SEED], dtype=np.uint64)
    for p in parts:
        if isinstance(p, str):
            vals = list(p.encode())
        else:
            vals = [int(p) & 0xFFFFFFFFFFFFFFFF]
        for v in vals:
            k = _splitmix64(k ^ np.uint64(v))
    return int(k[0])


def _raw(key: int, count: int, lane: int = 0) -> np.ndarray:
    """uint64 word i = splitmix64(key*golden + 2*i + lane) for i in [0,count)."""
    idx = np.arange(count, dtype=np.uint64)
    with np.errstate(over="ignore"):
        state = (np.uint64(key) + (idx * np.uint64(2) + np.uint64(lane)) *
                 np.uint64(0xD1342543DE82EF95)) & _M64
    return _splitmix64(_splitmix64(state))


def uniform_pm1(key: int, shape) -> np.ndarray:
    """fp32 uniform on [-1, 1) with 24-bit resolution."""
    n = int(np.prod(shape))
    u = _raw(key, n)
    v = (u >> np.uint64(40)).astype(np.float64) * (2.0 ** -23) - 1.0
    return v.astype(np.float32).reshape(shape)


def normal01(key: int, shape, scale: float = 1.0) -> np.ndarray:
    """fp32 N(0, scale^2) via Box-Muller in fp64."""
    n = int(np.prod(shape))
    u1 = ((_raw(key, n, 0) >> np.uint64(11)).astype(np.float64) + 1.0) * (2.0 ** -53)  # (0,1]
    u2 = (_raw(key, n, 1) >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)          # [0,1)
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return (z * scale).astype(np.float32).reshape(shape)


@dataclass(frozen=True)
class Layer:
    """One convolution layer: X[N,IH,IW,IC] * W[OC,FH,FW,IC] -> Y[N,OH,OW,OC]."""
    name: str
    N: int
    IH: int
    IW: int
    IC: int
    OC: int
    FH: int
    FW: int
    stride: int
    pad: int
    dist: str = "normal"     # "normal": X,G ~ N(0,1), W Kaiming-normal; "uniform": all U[-1,1)

    @property
    def OH(self) -> int:
        return (self.IH + 2 * self.pad - self.FH) // self.stride + 1

    @property
    def OW(self) -> int:
        return (self.IW + 2 * self.pad - self.FW) // self.stride + 1

    @property
    def M(self) -> int:
        return self.N * self.OH * self.OW

    @property
    def K(self) -> int:
        return self.FH * self.FW * self.IC

    @property
    def flops(self) -> int:
        """Nominal FLOP of one operator (padded taps counted): 2*M*OC*K."""
        return 2 * self.M * self.OC * self.K

    @property
    def in_range_share(self) -> float:
        """Share of the (output position, filter tap) pairs whose tap lies inside the image: the
        part of the nominal multiplies that is not a multiplication by padding."""
        rows = sum(1 for q in range(self.OH) for f in range(self.FH) if 0 <= q * self.stride - self.pad + f < self.IH)
        cols = sum(1 for q in range(self.OW) for f in range(self.FW) if 0 <= q * self.stride - self.pad + f < self.IW)
        return rows * cols / float(self.OH * self.OW * self.FH * self.FW)

    @property
    def effective_flops(self) -> float:
        """FLOP of one operator over in-range taps only (what a kernel that skips padding executes at least)."""
        return self.flops * self.in_range_share

    @property
    def x_shape(self):
        return (self.N, self.IH, self.IW, self.IC)

    @property
    def w_shape(self):
        return (self.OC, self.FH, self.FW, self.IC)

    @property
    def y_shape(self):
        return (self.N, self.OH, self.OW, self.OC)

    def with_batch(self, n: int) -> "Layer":
        return Layer(self.name + "@N%d" % n, n, self.IH, self.IW, self.IC, self.OC, self.FH,
                     self.FW, self.stride, self.pad, self.dist)


def make_inputs(layer: Layer, which=("X", "W", "G")):
    """Seeded tensors for a layer; returns a dict of fp32 numpy arrays."""
    out = {}
    for role in which:
        shape = {"X": layer.x_shape, "W": layer.w_shape, "G": layer.y_shape}[role]
        key = stream_key(layer.name.split("@")[0], layer.N, role)
        if layer.dist == "uniform":
            out[role] = uniform_pm1(key, shape)
        elif role == "W":
            out[role] = normal01(key, shape, scale=float(np.sqrt(2.0 / layer.K)))
        else:
            out[role] = normal01(key, shape)
    return out


# ---- the benchmark configurations (one Layer per operator triple) -----------------------
CFG1 = [Layer("C1", 4, 8, 8, 3, 16, 3, 3, 1, 1, dist="uniform")]
CFG2 = [Layer("C2", 128, 32, 32, 64, 128, 3, 3, 2, 1)]
CFG3 = [Layer("C3a", 128, 8, 8, 256, 256, 3, 3, 1, 1),
        Layer("C3b", 128, 4, 4, 512, 512, 3, 3, 1, 1),
        Layer("C3c", 128, 2, 2, 512, 512, 3, 3, 1, 1)]
CFG4 = [Layer("C4a", 128, 16, 16, 256, 64, 1, 1, 1, 0),
        Layer("C4b", 128, 16, 16, 256, 128, 3, 3, 1, 1),
        Layer("C4c", 128, 16, 16, 256, 32, 5, 5, 1, 2),
        Layer("C4d", 128, 32, 32, 64, 128, 1, 1, 2, 0)]


def _vgg16(n=128):
    chans = [(3, 64), (64, 64), "P", (64, 128), (128, 128), "P",
             (128, 256), (256, 256), (256, 256), "P",
             (256, 512), (512, 512), (512, 512), "P",
             (512, 512), (512, 512), (512, 512)]
    layers, hw, i = [], 32, 0
    for c in chans:
        if c == "P":
            hw //= 2
            continue
        i += 1
        layers.append(Layer("V%d" % i, n, hw, hw, c[0], c[1], 3, 3, 1, 1))
    return layers


CFG5 = _vgg16()
# stage ends after these layer indices (1-based) get a 2x2 max-pool in the VGG-16 chain
VGG_POOL_AFTER = (2, 4, 7, 10)

# Beyond the graded configurations: the paper's own batch size (512 images, Table I) and
# channel counts that are neither powers of two nor multiples of 32 everywhere (inception-style
# 96 / 160 / 192 / 48, where the paper notes its library loses ground, Sec. V).
CFG6 = [Layer("B1", 512, 8, 8, 256, 256, 3, 3, 1, 1),
        Layer("B2", 512, 16, 16, 128, 128, 3, 3, 1, 1),
        Layer("B3", 512, 4, 4, 512, 512, 3, 3, 1, 1),
        Layer("G1", 128, 16, 16, 192, 96, 1, 1, 1, 0),
        Layer("G2", 128, 16, 16, 96, 160, 3, 3, 1, 1),
        Layer("G3", 128, 8, 8, 160, 192, 3, 3, 1, 1),
        Layer("G4", 128, 16, 16, 192, 48, 5, 5, 1, 2),
        Layer("G5", 128, 8, 8, 48, 96, 3, 3, 1, 1)]

# Large feature maps (128x128 and up), the regime in which the paper concedes to the vendor
# library (Sec. IV): many tiles, no slicing of the reduction in forward / backward-data.
CFG7 = [Layer("L1", 8, 128, 128, 64, 64, 3, 3, 1, 1),
        Layer("L2", 4, 256, 256, 32, 32, 3, 3, 1, 1),
        Layer("L3", 8, 128, 128, 64, 128, 3, 3, 2, 1)]

# The distinct convolutions of a CIFAR-style ResNet-18 (3x3 stem, four stages of basic blocks,
# stride-2 3x3 and 1x1 shortcut convolutions between stages), batch 128: the other network family
# the paper trains (Sec. IV, Table III).  Repeated layers appear once.
CFG8 = [Layer("R1", 128, 32, 32, 3, 64, 3, 3, 1, 1),
        Layer("R2", 128, 32, 32, 64, 64, 3, 3, 1, 1),
        Layer("R3", 128, 32, 32, 64, 128, 3, 3, 2, 1),
        Layer("R3s", 128, 32, 32, 64, 128, 1, 1, 2, 0),
        Layer("R4", 128, 16, 16, 128, 128, 3, 3, 1, 1),
        Layer("R5", 128, 16, 16, 128, 256, 3, 3, 2, 1),
        Layer("R5s", 128, 16, 16, 128, 256, 1, 1, 2, 0),
        Layer("R6", 128, 8, 8, 256, 256, 3, 3, 1, 1),
        Layer("R7", 128, 8, 8, 256, 512, 3, 3, 2, 1),
        Layer("R7s", 128, 8, 8, 256, 512, 1, 1, 2, 0),
        Layer("R8", 128, 4, 4, 512, 512, 3, 3, 1, 1)]

# An AlexNet-shaped CIFAR layer set (the first network family of the paper's Table III; the paper does
# not print its layer list, so this is the usual CIFAR adaptation: 3x3 filters, 2x2 pooling after the
# first, second and fifth convolution), batch 128.  Synthetic stand-in like every other set.
CFG9 = [Layer("A1", 128, 32, 32, 3, 64, 3, 3, 1, 1),
        Layer("A2", 128, 16, 16, 64, 192, 3, 3, 1, 1),
        Layer("A3", 128, 8, 8, 192, 384, 3, 3, 1, 1),
        Layer("A4", 128, 8, 8, 384, 256, 3, 3, 1, 1),
        Layer("A5", 128, 8, 8, 256, 256, 3, 3, 1, 1)]

CONFIGS = {"cfg1": CFG1, "cfg2": CFG2, "cfg3": CFG3, "cfg4": CFG4, "cfg5": CFG5, "cfg6": CFG6,
           "cfg7": CFG7, "cfg8": CFG8, "cfg9": CFG9}


def all_layers():
    seen, out = set(), []
    for cfg in CONFIGS.values():
        for l in cfg:
            if l.name not in seen:
                seen.add(l.name)
                out.append(l)
    return out
