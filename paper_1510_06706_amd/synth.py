"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module computes nothing of the method on values: it fills arrays with
reproducible pseudo-random fp32 values and names the workloads (layer shapes of
the benchmark configurations, layer lists of the networks, graph descriptions)
together with the node extents that follow from them (``shapes``,
``graph_shapes``: bookkeeping for the product's harness, the GPU tests and the
benchmark).  The oracle works out its own extents, and its pin tests take their
shapes from ``tests/workloads.py``, not from here.  The values come from a
counter-based generator (SplitMix64 finaliser applied to ``seed, stream,
index``), so they do not depend on the numpy or torch version and can be
produced in any order.
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


# ---------------------------------------------------------------- layered networks
# 6 convolutional layers of width 40 with 3^3 kernels, a transfer function after each,
# 2^3 max-filters after the 2nd and 4th, 3 output images, 12^3 output patch => 26^3 input.
WIDTH = 40
CONFIG3_LAYERS = [
    ("conv", 1, WIDTH, (3, 3, 3)), ("transfer",),
    ("conv", WIDTH, WIDTH, (3, 3, 3)), ("transfer",), ("maxfilter", (2, 2, 2)),
    ("conv", WIDTH, WIDTH, (3, 3, 3)), ("transfer",),
    ("conv", WIDTH, WIDTH, (3, 3, 3)), ("transfer",), ("maxfilter", (2, 2, 2)),
    ("conv", WIDTH, WIDTH, (3, 3, 3)), ("transfer",),
    ("conv", WIDTH, 3, (3, 3, 3)), ("transfer",),
]
CONFIG3_INPUT = (1, 26, 26, 26)
CONFIG3_ETA = 1e-3
CONFIG3_SEED = 1003

# The same network as a max-filtering ConvNet that reproduces a sliding-window max-pooling
# ConvNet (Section 2, last paragraphs): every max-filter multiplies the sparsity of all
# later layers by its window, so the layers after the first filter have sparsity 2 and
# those after the second have sparsity 4.  Same 12^3 output patch => 43^3 input.
S2, S4 = (2, 2, 2), (4, 4, 4)
CONFIG3_SPARSE_LAYERS = [
    ("conv", 1, WIDTH, (3, 3, 3)), ("transfer",),
    ("conv", WIDTH, WIDTH, (3, 3, 3)), ("transfer",), ("maxfilter", (2, 2, 2)),
    ("conv", WIDTH, WIDTH, (3, 3, 3), S2), ("transfer",),
    ("conv", WIDTH, WIDTH, (3, 3, 3), S2), ("transfer",), ("maxfilter", (2, 2, 2), S2),
    ("conv", WIDTH, WIDTH, (3, 3, 3), S4), ("transfer",),
    ("conv", WIDTH, 3, (3, 3, 3), S4), ("transfer",),
]
CONFIG3_SPARSE_INPUT = (1, 43, 43, 43)

ONES = (1, 1, 1)


def _opt(spec, i, default):
    return spec[i] if len(spec) > i else default


def shapes(layers, in_shape):
    """Node shapes [maps, z, y, x] before every layer and after the last."""
    out = [tuple(in_shape)]
    for spec in layers:
        m, n = out[-1][0], out[-1][1:]
        if spec[0] == "conv":
            assert spec[1] == m
            out.append((spec[2],) + tuple(a - s * (b - 1) for a, b, s in zip(n, spec[3], _opt(spec, 4, ONES))))
        elif spec[0] == "transfer":
            out.append(out[-1])
        elif spec[0] == "maxfilter":
            out.append((m,) + tuple(a - s * (b - 1) for a, b, s in zip(n, spec[1], _opt(spec, 2, ONES))))
        elif spec[0] == "maxpool":
            assert all(a % b == 0 for a, b in zip(n, spec[1])), "max-pooling needs n divisible by p"
            out.append((m,) + tuple(a // b for a, b in zip(n, spec[1])))
        else:
            raise ValueError(spec)
    return out


def synthetic_params(layers, seed):
    """fp32 kernels uniform[-1,1) * sqrt(6 / (f k^3)) and biases uniform[-0.1,0.1), seeded per layer."""
    params = []
    for l, spec in enumerate(layers):
        if spec[0] == "conv":
            f, fo, k = spec[1:4]
            scale = float(np.sqrt(6.0 / (f * int(np.prod(k)))))
            params.append({"w": uniform_pm1(seed + 17 * l, STREAM_KERNEL, (fo, f) + tuple(k), scale)})
        elif spec[0] == "transfer":
            maps = [s for s in layers[:l] if s[0] == "conv"][-1][2]
            params.append({"b": uniform_pm1(seed + 17 * l, STREAM_BIAS, (maps,), 0.1)})
        else:
            params.append(None)
    return params


def net_tensors(layers, in_shape, seed):
    """(input, target, params) of a layered net: input uniform[-1,1), target uniform[0,1)."""
    x = uniform_pm1(seed, STREAM_IMAGE, in_shape)
    target = uniform_01(seed, STREAM_TARGET, shapes(layers, in_shape)[-1])
    return x, target, synthetic_params(layers, seed)


def config3_tensors():
    return net_tensors(CONFIG3_LAYERS, CONFIG3_INPUT, CONFIG3_SEED)


# The paper's 2D benchmark network (Section 6, scalability experiments): 6 convolutional layers
# with 11x11 kernels, a rectifier after each, 2x2 max-filters after the 2nd and 4th
# (CTMCTMCTCTCTCT as printed: the filters follow the first two transfer layers), 48x48 output
# patch => 110x110 input.  2D is the special case with one extent equal to 1.  Width 40.
K11, M2 = (1, 11, 11), (1, 2, 2)
CONFIG2D_LAYERS = [
    ("conv", 1, WIDTH, K11), ("transfer",), ("maxfilter", M2),
    ("conv", WIDTH, WIDTH, K11), ("transfer",), ("maxfilter", M2),
    ("conv", WIDTH, WIDTH, K11), ("transfer",),
    ("conv", WIDTH, WIDTH, K11), ("transfer",),
    ("conv", WIDTH, WIDTH, K11), ("transfer",),
    ("conv", WIDTH, 3, K11), ("transfer",),
]
CONFIG2D_INPUT = (1, 1, 110, 110)
CONFIG2D_SEED = 1006


def config2d_tensors():
    return net_tensors(CONFIG2D_LAYERS, CONFIG2D_INPUT, CONFIG2D_SEED)


def config3_sparse_tensors():
    return net_tensors(CONFIG3_SPARSE_LAYERS, CONFIG3_SPARSE_INPUT, CONFIG3_SEED + 1)


# ---------------------------------------------------------------- general computation graphs
# Nodes are groups of images, edges are bundles of operations between two groups:
#   ("conv", name, src, dst, f_out, k[, s]) | ("transfer", name, src, dst[, fn])
#   ("maxfilter", name, src, dst, win[, s]) | ("maxpool", name, src, dst, p)
# A node's image is the sum of its incoming edges' outputs, so all of them must agree in shape.
def graph_shapes(graph):
    """Shape [maps, z, y, x] of every node, by propagating the input shapes along the edges."""
    shape = {n: tuple(s) for n, s in graph["inputs"].items()}
    pending = list(graph["edges"])
    while pending:
        rest = []
        for e in pending:
            kind, name, src, dst = e[:4]
            if src not in shape:
                rest.append(e)
                continue
            m, n = shape[src][0], shape[src][1:]
            if kind == "conv":
                out = (e[4],) + tuple(a - s * (b - 1) for a, b, s in zip(n, e[5], _opt(e, 6, ONES)))
            elif kind == "transfer":
                out = shape[src]
            elif kind == "maxfilter":
                out = (m,) + tuple(a - s * (b - 1) for a, b, s in zip(n, e[4], _opt(e, 5, ONES)))
            elif kind == "maxpool":
                assert all(a % b == 0 for a, b in zip(n, e[4])), "max-pooling needs n divisible by p"
                out = (m,) + tuple(a // b for a, b in zip(n, e[4]))
            else:
                raise ValueError(e)
            assert min(out) >= 1, ("edge %s leaves no voxels" % name)
            assert shape.setdefault(dst, out) == out, ("edges into %s disagree in shape" % dst)
        if len(rest) == len(pending):
            raise ValueError("graph has an edge whose source is never produced")
        pending = rest
    return shape


def graph_params(graph, seed):
    """fp32 parameters per edge name, same distributions as ``synthetic_params``."""
    shape = graph_shapes(graph)
    params = {}
    for i, e in enumerate(graph["edges"]):
        kind, name, src = e[:3]
        if kind == "conv":
            f, fo, k = shape[src][0], e[4], tuple(e[5])
            scale = float(np.sqrt(6.0 / (f * int(np.prod(k)))))
            params[name] = {"w": uniform_pm1(seed + 17 * i, STREAM_KERNEL, (fo, f) + k, scale)}
        elif kind == "transfer":
            params[name] = {"b": uniform_pm1(seed + 17 * i, STREAM_BIAS, (shape[src][0],), 0.1)}
    return params


def graph_tensors(graph, seed):
    """(inputs, targets, params): inputs uniform[-1,1), targets uniform[0,1) per output node."""
    shape = graph_shapes(graph)
    inputs = {n: uniform_pm1(seed + 3 * i, STREAM_IMAGE, s) for i, (n, s) in enumerate(sorted(graph["inputs"].items()))}
    targets = {n: uniform_01(seed + 5 * i, STREAM_TARGET, shape[n]) for i, n in enumerate(graph["outputs"])}
    return inputs, targets, graph_params(graph, seed)


def multiscale_graph(width=8, n=24):
    """A small multi-scale net: after a shared first layer three branches with sparsity 1, 2 and
    3 (fields of view 5, 5 and 5 voxels wide, sampled at different scales) converge on one node."""
    k3, k2 = (3, 3, 3), (2, 2, 2)
    return {
        "inputs": {"x": (1, n, n, n)},
        "edges": [
            ("conv", "c0", "x", "a", width, k3), ("transfer", "t0", "a", "a1"),
            # fine branch: two dense convolutions
            ("conv", "c1", "a1", "b", width, k3), ("transfer", "t1", "b", "b1"),
            ("conv", "c2", "b1", "c", width, k3),
            # skip branch: one convolution with sparsity 2
            ("conv", "c3", "a1", "c", width, k3, (2, 2, 2)),
            # coarse branch: max-filter, then a convolution with sparsity 3
            ("maxfilter", "m0", "a1", "m", k2),
            ("conv", "c4", "m", "c", width, k2, (3, 3, 3)),
            ("transfer", "t2", "c", "c1", "tanh"),
            ("conv", "c5", "c1", "o", 2, k3), ("transfer", "t3", "o", "y", "logistic"),
            # a second output taken from the fine branch alone
            ("conv", "c6", "b1", "p", 1, k3), ("transfer", "t4", "p", "y2", "logistic"),
        ],
        "outputs": ["y", "y2"],
    }
