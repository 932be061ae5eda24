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


def shapes(layers, in_shape):
    """Node shapes [maps, z, y, x] before every layer and after the last."""
    out = [tuple(in_shape)]
    for spec in layers:
        m, n = out[-1][0], out[-1][1:]
        if spec[0] == "conv":
            assert spec[1] == m
            out.append((spec[2],) + tuple(a - b + 1 for a, b in zip(n, spec[3])))
        elif spec[0] == "transfer":
            out.append(out[-1])
        elif spec[0] == "maxfilter":
            out.append((m,) + tuple(a - b + 1 for a, b in zip(n, spec[1])))
    return out


def synthetic_params(layers, seed):
    """fp32 kernels uniform[-1,1) * sqrt(6 / (f k^3)) and biases uniform[-0.1,0.1), seeded per layer."""
    params = []
    for l, spec in enumerate(layers):
        if spec[0] == "conv":
            _, f, fo, k = spec
            scale = float(np.sqrt(6.0 / (f * int(np.prod(k)))))
            params.append({"w": synth.uniform_pm1(seed + 17 * l, synth.STREAM_KERNEL, (fo, f) + tuple(k), scale)})
        elif spec[0] == "transfer":
            maps = [s for s in layers[:l] if s[0] == "conv"][-1][2]
            params.append({"b": synth.uniform_pm1(seed + 17 * l, synth.STREAM_BIAS, (maps,), 0.1)})
        else:
            params.append(None)
    return params


def config3_tensors():
    x = synth.uniform_pm1(CONFIG3_SEED, synth.STREAM_IMAGE, CONFIG3_INPUT)
    out_shape = shapes(CONFIG3_LAYERS, CONFIG3_INPUT)[-1]
    target = synth.uniform_01(CONFIG3_SEED, synth.STREAM_TARGET, out_shape)
    return x, target, synthetic_params(CONFIG3_LAYERS, CONFIG3_SEED)


class Net:
    """Device-side state of a layered net: plans per convolution, parameters as CUDA tensors."""

    def __init__(self, layers, in_shape, params, mode="auto", device="cuda:0"):
        import torch
        self.layers = list(layers)
        self.shapes = shapes(layers, in_shape)
        self.device = device
        self.params = [None if p is None else {k: torch.from_numpy(np.ascontiguousarray(v)).to(device)
                                               for k, v in p.items()} for p in params]
        self.plans = []
        for l, spec in enumerate(self.layers):
            if spec[0] == "conv":
                m = mode[l] if isinstance(mode, (list, tuple)) else mode
                self.plans.append(znn.Plan(spec[1], spec[2], self.shapes[l][1:], spec[3], m))
            else:
                self.plans.append(None)

    def modes(self):
        return [None if p is None else p.mode for p in self.plans]

    def forward(self, x):
        acts, aux = [x], [None] * len(self.layers)
        for l, spec in enumerate(self.layers):
            a = acts[-1]
            if spec[0] == "conv":
                y = self.plans[l].fwd(a, self.params[l]["w"])
            elif spec[0] == "transfer":
                y = znn.transfer_fwd(a, self.params[l]["b"])
            else:
                y, aux[l] = znn.maxfilter3d_fwd(a, spec[1])
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
            if spec[0] == "conv":
                grads[l] = {"w": self.plans[l].wgrad(acts[l], g)}
                g = self.plans[l].bwd(g, self.params[l]["w"]) if l > 0 else None
            elif spec[0] == "transfer":
                g = znn.transfer_bwd(g, acts[l + 1])
                grads[l] = {"b": znn.bias_grad(g)}
            else:
                g = znn.maxfilter3d_bwd(g, aux[l], self.shapes[l][1:], spec[1])
        return grads

    def train_round(self, x, target, eta, record=None):
        acts, aux = self.forward(x)
        gout = znn.square_loss_grad(acts[-1], target)
        grads = self.backward(acts, aux, gout, record)
        for p, g in zip(self.params, grads):
            if p is not None:
                for k in p:
                    znn.sgd_update(p[k], g[k], eta)
        return acts, aux, gout, grads
