"""Seeded synthetic inputs and layer-shape tables for the conv2d hot path.

This module holds no convolution arithmetic.  It only (a) names the layer
geometries of the convnets the paper benchmarks (abstract and Sec. 3.4: AlexNet,
VGG, Overfeat, GoogLeNet) and (b) fills tensors from a counter-based generator so
that the CPU oracle and the HIP library can be fed the very same bytes.

Generator: SplitMix64 evaluated at a counter (element index), so element i of a
tensor depends on (seed, i) only and tensors can be produced in chunks.
  U(a,b): top 24 bits of the 64-bit word scaled to [0,1), then affine.
  N(0,1): Box-Muller on the words at counters 2i and 2i+1 (fp64, rounded to fp32).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22

BASE_SEED = 160604884


def _splitmix64(seed: int, idx: np.ndarray) -> np.ndarray:
    """64-bit SplitMix64 output for counters idx (uint64 array)."""
    with np.errstate(over="ignore"):
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + (idx + np.uint64(1)) * _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def _unit(seed: int, idx: np.ndarray) -> np.ndarray:
    """fp64 values in [0,1) with 24 random bits."""
    return (_splitmix64(seed, idx) >> np.uint64(40)).astype(np.float64) * (1.0 / (1 << 24))


def uniform(shape, seed: int, lo: float = -1.0, hi: float = 1.0) -> np.ndarray:
    """fp32 tensor ~ U(lo,hi), C-contiguous."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    for s in range(0, n, _CHUNK):
        e = min(n, s + _CHUNK)
        idx = np.arange(s, e, dtype=np.uint64)
        out[s:e] = (lo + (hi - lo) * _unit(seed, idx)).astype(np.float32)
    return out.reshape(shape)


def normal(shape, seed: int, std: float = 1.0) -> np.ndarray:
    """fp32 tensor ~ N(0, std^2), C-contiguous."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    for s in range(0, n, _CHUNK):
        e = min(n, s + _CHUNK)
        idx = np.arange(s, e, dtype=np.uint64)
        u1 = _unit(seed, idx * np.uint64(2)) + 2.0 ** -25
        u2 = _unit(seed, idx * np.uint64(2) + np.uint64(1))
        g = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        out[s:e] = (std * g).astype(np.float32)
    return out.reshape(shape)


def dyadic(shape, seed: int, denom: int = 8, span: int = 16) -> np.ndarray:
    """fp32 tensor of multiples of 1/denom in [-span/denom, span/denom]: sums and
    products of such values are exact in fp64, which exact-equality tests rely on."""
    n = int(np.prod(shape))
    idx = np.arange(n, dtype=np.uint64)
    k = (_splitmix64(seed, idx) >> np.uint64(33)).astype(np.int64) % (2 * span + 1) - span
    return (k.astype(np.float64) / denom).astype(np.float32).reshape(shape)


@dataclass(frozen=True)
class Layer:
    """Geometry of one conv layer: input N x C x H x W, K filters of R x S."""
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

    def desc(self) -> Tuple[int, ...]:
        return (self.N, self.C, self.H, self.W, self.K, self.R, self.S,
                self.stride, self.stride, self.pad, self.pad)

    def with_batch(self, n: int) -> "Layer":
        return Layer(self.name, n, self.C, self.H, self.W, self.K, self.R, self.S,
                     self.stride, self.pad)


def _vgg16(n: int) -> List[Layer]:
    plan = [("conv1_1", 3, 224, 64), ("conv1_2", 64, 224, 64),
            ("conv2_1", 64, 112, 128), ("conv2_2", 128, 112, 128),
            ("conv3_1", 128, 56, 256), ("conv3_2", 256, 56, 256), ("conv3_3", 256, 56, 256),
            ("conv4_1", 256, 28, 512), ("conv4_2", 512, 28, 512), ("conv4_3", 512, 28, 512),
            ("conv5_1", 512, 14, 512), ("conv5_2", 512, 14, 512), ("conv5_3", 512, 14, 512)]
    return [Layer(nm, n, c, hw, hw, k, 3, 3, 1, 1) for nm, c, hw, k in plan]


def config_layers(config: int, batch: int | None = None) -> List[Layer]:
    """Layer lists of the five benchmark configurations (index 0..4).  Every layer
    is an independent synthetic layer at its stated input shape."""
    if config == 0:
        n = batch or 2
        return [Layer("tiny", n, 3, 16, 16, 8, 3, 3, 1, 1)]
    if config == 1:  # AlexNet-shaped
        n = batch or 128
        return [Layer("conv1", n, 3, 224, 224, 64, 11, 11, 4, 2),
                Layer("conv2", n, 64, 27, 27, 192, 5, 5, 1, 2),
                Layer("conv3", n, 192, 13, 13, 384, 3, 3, 1, 1),
                Layer("conv4", n, 384, 13, 13, 256, 3, 3, 1, 1),
                Layer("conv5", n, 256, 13, 13, 256, 3, 3, 1, 1)]
    if config == 2:  # VGG-16
        return _vgg16(batch or 64)
    if config == 3:  # GoogLeNet inception module on 192x28x28
        n = batch or 128
        return [Layer("1x1", n, 192, 28, 28, 64, 1, 1, 1, 0),
                Layer("3x3_reduce", n, 192, 28, 28, 96, 1, 1, 1, 0),
                Layer("3x3", n, 96, 28, 28, 128, 3, 3, 1, 1),
                Layer("5x5_reduce", n, 192, 28, 28, 16, 1, 1, 1, 0),
                Layer("5x5", n, 16, 28, 28, 32, 5, 5, 1, 2),
                Layer("pool_proj", n, 192, 28, 28, 32, 1, 1, 1, 0)]
    if config == 4:  # Overfeat-fast-shaped
        n = batch or 128
        return [Layer("conv1", n, 3, 231, 231, 96, 11, 11, 4, 0),
                Layer("conv2", n, 96, 24, 24, 256, 5, 5, 1, 0),
                Layer("conv3", n, 256, 12, 12, 512, 3, 3, 1, 1),
                Layer("conv4", n, 512, 12, 12, 1024, 3, 3, 1, 1),
                Layer("conv5", n, 1024, 12, 12, 1024, 3, 3, 1, 1)]
    raise ValueError("config must be 0..4")


def layer_seed(config: int, layer: int, tensor: int) -> int:
    """tensor: 0 x, 1 w, 2 b, 3 dy."""
    return BASE_SEED + 1000 * (config + 1) + 10 * layer + tensor


def layer_tensors(config: int, layer_idx: int, L: Layer, out_hw: Tuple[int, int]
                  ) -> Dict[str, np.ndarray]:
    """x, w, b, dy for one layer, with the value distributions of its config:
    config 0: x,w,b ~ U(-1,1); others: x ~ N(0,1), w ~ N(0, 2/(C R S)) (He, fan-in),
    b ~ U(-0.1,0.1).  dy ~ N(0,1) everywhere.  out_hw = (P, Q) of the layer."""
    P, Q = out_hw
    sx, sw, sb, sdy = (layer_seed(config, layer_idx, t) for t in range(4))
    if config == 0:
        x = uniform((L.N, L.C, L.H, L.W), sx)
        w = uniform((L.K, L.C, L.R, L.S), sw)
        b = uniform((L.K,), sb)
    else:
        x = normal((L.N, L.C, L.H, L.W), sx)
        w = normal((L.K, L.C, L.R, L.S), sw, std=float(np.sqrt(2.0 / (L.C * L.R * L.S))))
        b = uniform((L.K,), sb, -0.1, 0.1)
    dy = normal((L.N, L.K, P, Q), sdy)
    return {"x": x, "w": w, "b": b, "dy": dy}
