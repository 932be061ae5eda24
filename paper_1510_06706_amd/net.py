"""One training round of a layered ConvNet driven through the C ABI (config-3 harness).

This module only sequences library calls (Section 3 of the paper: forward pass,
loss gradient, backward pass, gradients, update); every arithmetic step runs in
libznn's kernels.  It also names the benchmark network and builds its seeded
synthetic parameters.
"""
from __future__ import annotations

import numpy as np

from . import binding as znn
from . import synth

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
            params.append({"w": synth.uniform_pm1(seed + 17 * l, synth.STREAM_KERNEL, (fo, f) + tuple(k), scale)})
        elif spec[0] == "transfer":
            maps = [s for s in layers[:l] if s[0] == "conv"][-1][2]
            params.append({"b": synth.uniform_pm1(seed + 17 * l, synth.STREAM_BIAS, (maps,), 0.1)})
        else:
            params.append(None)
    return params


def net_tensors(layers, in_shape, seed):
    """(input, target, params) of a layered net: input uniform[-1,1), target uniform[0,1)."""
    x = synth.uniform_pm1(seed, synth.STREAM_IMAGE, in_shape)
    target = synth.uniform_01(seed, synth.STREAM_TARGET, shapes(layers, in_shape)[-1])
    return x, target, synthetic_params(layers, seed)


def config3_tensors():
    return net_tensors(CONFIG3_LAYERS, CONFIG3_INPUT, CONFIG3_SEED)


def config3_sparse_tensors():
    return net_tensors(CONFIG3_SPARSE_LAYERS, CONFIG3_SPARSE_INPUT, CONFIG3_SEED + 1)


class Net:
    """Device-side state of a layered net: plans per convolution, parameters as CUDA tensors.

    ``mode`` is "direct", "fft", "auto" (cached autotuner choice or cost model), a list with
    one entry per layer, or "tuned": every convolutional layer is timed as a whole round in
    the three strategies direct / FFT / FFT with memoized spectra (Section 4) and takes the
    fastest one whose buffers fit ``memory_budget`` bytes (per layer; None = no limit).
    """

    def __init__(self, layers, in_shape, params, mode="auto", device="cuda:0", memory_budget=None):
        import torch
        self.layers = list(layers)
        self.shapes = shapes(layers, in_shape)
        self.device = device
        self.params = [None if p is None else {k: torch.from_numpy(np.ascontiguousarray(v)).to(device)
                                               for k, v in p.items()} for p in params]
        self.plans = []
        self.strategy = [None] * len(self.layers)
        self.tuning = {}
        for l, spec in enumerate(self.layers):
            if spec[0] == "conv":
                m = mode[l] if isinstance(mode, (list, tuple)) else mode
                sp = _opt(spec, 4, ONES)
                if m == "tuned":
                    m, ms, nbytes = znn.autotune_round(spec[1], spec[2], self.shapes[l][1:], spec[3],
                                                       memory_budget, sp, device)
                    self.tuning[l] = (m, ms, nbytes)
                plan = znn.Plan(spec[1], spec[2], self.shapes[l][1:], spec[3], "fft" if m == "fft_memo" else m, sp)
                if m == "fft_memo":
                    plan.enable_memo(device)
                self.strategy[l] = m
                self.plans.append(plan)
            else:
                self.plans.append(None)

    def modes(self):
        return [None if p is None else p.mode for p in self.plans]

    def forward(self, x):
        acts, aux = [x], [None] * len(self.layers)
        for l, spec in enumerate(self.layers):
            a = acts[-1]
            if spec[0] == "conv" and self.strategy[l] == "fft_memo":
                self.plans[l].prepare_kernels(self.params[l]["w"])      # once per round: w changes every update
                y = self.plans[l].fwd(a, None)
            elif spec[0] == "conv":
                y = self.plans[l].fwd(a, self.params[l]["w"])
            elif spec[0] == "transfer":
                y = znn.transfer_fwd(a, self.params[l]["b"], _opt(spec, 1, "rectify"))
            elif spec[0] == "maxfilter":
                y, aux[l] = znn.maxfilter3d_fwd(a, spec[1], _opt(spec, 2, ONES))
            else:
                y, aux[l] = znn.maxpool3d_fwd(a, spec[1])
            acts.append(y)
        return acts, aux

    def backward(self, acts, aux, gout, record=None):
        """`record`, if a list, receives (layer, gradient arriving at that layer's output)."""
        grads = [None] * len(self.layers)
        g = gout
        for l in range(len(self.layers) - 1, -1, -1):
            spec = self.layers[l]
            if record is not None:
                record.append((l, g))
            if spec[0] == "conv" and self.strategy[l] == "fft_memo" and l > 0:
                # backward first: it leaves the spectra of g next to those of the forward input
                g = self.plans[l].bwd(g, None)
                grads[l] = {"w": self.plans[l].wgrad_memo(device=self.device)}
            elif spec[0] == "conv":
                grads[l] = {"w": self.plans[l].wgrad(acts[l], g)}
                g = self.plans[l].bwd(g, self.params[l]["w"]) if l > 0 else None
            elif spec[0] == "transfer":
                g = znn.transfer_bwd(g, acts[l + 1], _opt(spec, 1, "rectify"))
                grads[l] = {"b": znn.bias_grad(g)}
            elif spec[0] == "maxfilter":
                g = znn.maxfilter3d_bwd(g, aux[l], self.shapes[l][1:], spec[1], _opt(spec, 2, ONES))
            else:
                g = znn.maxpool3d_bwd(g, aux[l], self.shapes[l][1:], spec[1])
        return grads

    def train_round(self, x, target, eta, record=None, loss="square"):
        acts, aux = self.forward(x)
        gout = znn.loss_grad(acts[-1], target, loss)
        grads = self.backward(acts, aux, gout, record)
        for p, g in zip(self.params, grads):
            if p is not None:
                for k in p:
                    znn.sgd_update(p[k], g[k], eta)
        return acts, aux, gout, grads
