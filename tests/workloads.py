"""Test-side descriptions of small networks and graphs for the oracle's pin tests.

The oracle's tests must not lean on the product package for anything but the seeded value
generator (``synth.uniform_pm1`` / ``uniform_01``), so the shapes and parameter sets they need
are worked out here, independently of ``paper_1510_06706_amd.net`` / ``graph``.
Layer specs:  ("conv", f, f', k[, s]) | ("transfer"[, fn]) | ("maxfilter", win[, s]) | ("maxpool", p)
"""
import numpy as np

from paper_1510_06706_amd.synth import uniform_01, uniform_pm1

KERNEL_STREAM, BIAS_STREAM, IMAGE_STREAM, TARGET_STREAM = 1, 4, 0, 3


def _sparsity(spec, i):
    return tuple(spec[i]) if len(spec) > i else (1, 1, 1)


def _after(kind, spec, maps, n):
    """Shape [maps, z, y, x] behind one layer (Section 2: valid sizes n - s (k - 1); pooling n / p)."""
    if kind == "conv":
        s = _sparsity(spec, 4)
        return (spec[2],) + tuple(n[d] - s[d] * (spec[3][d] - 1) for d in range(3))
    if kind == "transfer":
        return (maps,) + tuple(n)
    if kind == "maxfilter":
        s = _sparsity(spec, 2)
        return (maps,) + tuple(n[d] - s[d] * (spec[1][d] - 1) for d in range(3))
    if kind == "maxpool":
        assert all(n[d] % spec[1][d] == 0 for d in range(3))
        return (maps,) + tuple(n[d] // spec[1][d] for d in range(3))
    raise ValueError(spec)


def layer_shapes(layers, in_shape):
    out = [tuple(in_shape)]
    for spec in layers:
        out.append(_after(spec[0], spec, out[-1][0], out[-1][1:]))
    return out


def layer_params(layers, seed):
    """float64 kernels uniform[-1,1) sqrt(6 / (f k^3)) and biases uniform[-0.1,0.1), one seed per layer."""
    params, maps = [], None
    for l, spec in enumerate(layers):
        if spec[0] == "conv":
            f, fo, k = spec[1], spec[2], tuple(spec[3])
            maps = fo
            scale = np.sqrt(6.0 / (f * int(np.prod(k))))
            params.append({"w": uniform_pm1(seed + 17 * l, KERNEL_STREAM, (fo, f) + k).astype(np.float64) * scale})
        elif spec[0] == "transfer":
            params.append({"b": uniform_pm1(seed + 17 * l, BIAS_STREAM, (maps,)).astype(np.float64) * 0.1})
        else:
            params.append(None)
    return params


def net_tensors(layers, in_shape, seed):
    x = uniform_pm1(seed, IMAGE_STREAM, in_shape).astype(np.float64)
    t = uniform_01(seed, TARGET_STREAM, layer_shapes(layers, in_shape)[-1]).astype(np.float64)
    return x, t, layer_params(layers, seed)


# Graph edges: ("conv", name, src, dst, f', k[, s]) | ("transfer", name, src, dst[, fn])
#              ("maxfilter", name, src, dst, win[, s]) | ("maxpool", name, src, dst, p)
def graph_shapes(graph):
    shape = {n: tuple(s) for n, s in graph["inputs"].items()}
    todo = list(graph["edges"])
    while todo:
        later = []
        for e in todo:
            kind, _, src, dst = e[:4]
            if src not in shape:
                later.append(e)
                continue
            spec = {"conv": lambda: ("conv", shape[src][0], e[4], e[5]) + tuple(e[6:7]),
                    "transfer": lambda: ("transfer",),
                    "maxfilter": lambda: ("maxfilter", e[4]) + tuple(e[5:6]),
                    "maxpool": lambda: ("maxpool", e[4])}[kind]()
            got = _after(kind, spec, shape[src][0], shape[src][1:])
            assert shape.setdefault(dst, got) == got
        assert len(later) < len(todo)
        todo = later
    return shape


def graph_tensors(graph, seed):
    """(inputs, targets, params) in float64 for a graph description."""
    shape = graph_shapes(graph)
    inputs = {n: uniform_pm1(seed + 3 * i, IMAGE_STREAM, s).astype(np.float64)
              for i, (n, s) in enumerate(sorted(graph["inputs"].items()))}
    targets = {n: uniform_01(seed + 5 * i, TARGET_STREAM, shape[n]).astype(np.float64)
               for i, n in enumerate(graph["outputs"])}
    params = {}
    for i, e in enumerate(graph["edges"]):
        kind, name, src = e[:3]
        if kind == "conv":
            f, fo, k = shape[src][0], e[4], tuple(e[5])
            scale = np.sqrt(6.0 / (f * int(np.prod(k))))
            params[name] = {"w": uniform_pm1(seed + 17 * i, KERNEL_STREAM, (fo, f) + k).astype(np.float64) * scale}
        elif kind == "transfer":
            params[name] = {"b": uniform_pm1(seed + 17 * i, BIAS_STREAM, (shape[src][0],)).astype(np.float64) * 0.1}
    return inputs, targets, params


def multiscale_graph(width=2, n=11):
    """Shared first layer, then three branches (dense, sparsity 2, max-filter + sparsity 3) that converge
    on one node; a second output hangs off the dense branch."""
    k3, k2 = (3, 3, 3), (2, 2, 2)
    return {
        "inputs": {"x": (1, n, n, n)},
        "edges": [
            ("conv", "c0", "x", "a", width, k3), ("transfer", "t0", "a", "a1"),
            ("conv", "c1", "a1", "b", width, k3), ("transfer", "t1", "b", "b1"),
            ("conv", "c2", "b1", "c", width, k3),
            ("conv", "c3", "a1", "c", width, k3, (2, 2, 2)),
            ("maxfilter", "m0", "a1", "m", k2),
            ("conv", "c4", "m", "c", width, k2, (3, 3, 3)),
            ("transfer", "t2", "c", "c1", "tanh"),
            ("conv", "c5", "c1", "o", 2, k3), ("transfer", "t3", "o", "y", "logistic"),
            ("conv", "c6", "b1", "p", 1, k3), ("transfer", "t4", "p", "y2", "logistic"),
        ],
        "outputs": ["y", "y2"],
    }
