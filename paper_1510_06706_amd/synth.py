"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds no arithmetic of the method itself: it only fills arrays
with reproducible pseudo-random fp32 values and names the layer shapes of the
benchmark configurations.  The values come from a counter-based generator
(SplitMix64 finaliser applied to ``seed, stream, index``), so they do not
depend on the numpy or torch version and can be produced in any order.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Tuple

import numpy as np

STREAM_IMAGE = 0
STREAM_KERNEL = 1
STREAM_OUTGRAD = 2
STREAM_TARGET = 3
STREAM_BIAS = 4

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def raw_bits(seed: int, stream: int, count: int, offset: int = 0) -> np.ndarray:
    """24 pseudo-random bits per element as uint32, for indices offset..offset+count."""
    with np.errstate(over="ignore"):
        base = _mix(np.array([(int(seed) * 0x9E3779B97F4A7C15 + int(stream) * 0xD1B54A32D192ED03
                               + 0x2545F4914F6CDD1D) & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64))[0]
        idx = np.arange(offset, offset + count, dtype=np.uint64)
        z = _mix(base + (idx + np.uint64(1)) * np.uint64(0x9E3779B97F4A7C15))
    return (z >> np.uint64(40)).astype(np.uint32)


def uniform_pm1(seed: int, stream: int, shape, scale: float = 1.0) -> np.ndarray:
    """fp32 values uniform on the grid {m / 2^23 : -2^23 <= m < 2^23}, times ``scale``."""
    count = int(np.prod(shape))
    out = np.empty(count, dtype=np.float32)
    step = 1 << 24
    for lo in range(0, count, step):
        c = min(step, count - lo)
        bits = raw_bits(seed, stream, c, lo).astype(np.int64)
        out[lo:lo + c] = ((bits - (1 << 23)).astype(np.float32) / np.float32(1 << 23))
    if scale != 1.0:
        out *= np.float32(scale)
    return out.reshape(shape)


def uniform_01(seed: int, stream: int, shape) -> np.ndarray:
    """fp32 values uniform on the grid {m / 2^24 : 0 <= m < 2^24}."""
    count = int(np.prod(shape))
    bits = raw_bits(seed, stream, count)
    return (bits.astype(np.float32) / np.float32(1 << 24)).reshape(shape)


@dataclass(frozen=True)
class LayerShape:
    """One fully connected convolutional layer: f input nodes, f' output nodes."""
    name: str
    fan_in: int
    fan_out: int
    image: Tuple[int, int, int]      # n  (z, y, x)
    kernel: Tuple[int, int, int]     # k  (z, y, x)
    kernel_scale: float = 1.0
    seed: int = 0
    sparsity: Tuple[int, int, int] = (1, 1, 1)   # s (z, y, x): taps are s voxels apart

    @property
    def out(self) -> Tuple[int, int, int]:
        return tuple(n - s * (k - 1) for n, k, s in zip(self.image, self.kernel, self.sparsity))

    @property
    def macs(self) -> int:
        return self.fan_in * self.fan_out * int(np.prod(self.out)) * int(np.prod(self.kernel))

    @property
    def out_voxels(self) -> int:
        return self.fan_out * int(np.prod(self.out))


# The benchmark configurations (single-layer ones).  Shapes follow the wide
# 3D and 2D networks of the paper's experiments; values are synthetic.
CONFIG1 = LayerShape("c1_1to4_16cube_k3", 1, 4, (16, 16, 16), (3, 3, 3), 1.0, 1001)
CONFIG2 = LayerShape("c2_40to40_64cube_k5", 40, 40, (64, 64, 64), (5, 5, 5),
                     1.0 / float(np.sqrt(40 * 125)), 1002)
CONFIG4 = LayerShape("c4_80to80_256sq_k11", 80, 80, (1, 256, 256), (1, 11, 11), 1.0, 1004)
CONFIG5 = LayerShape("c5_120to120_96cube_k7", 120, 120, (96, 96, 96), (7, 7, 7),
                     1.0 / float(np.sqrt(120 * 343)), 1005)


def layer_tensors(cfg: LayerShape, seed: int | None = None):
    """(in, w, gout) fp32 arrays for a layer, values uniform in [-1, 1) (kernels scaled)."""
    s = cfg.seed if seed is None else seed
    inp = uniform_pm1(s, STREAM_IMAGE, (cfg.fan_in,) + tuple(cfg.image))
    w = uniform_pm1(s, STREAM_KERNEL, (cfg.fan_out, cfg.fan_in) + tuple(cfg.kernel), cfg.kernel_scale)
    gout = uniform_pm1(s, STREAM_OUTGRAD, (cfg.fan_out,) + tuple(cfg.out))
    return inp, w, gout
