"""Float64 reference of one training round of a layered ConvNet (TEST INFRASTRUCTURE ONLY).

The round follows Section 3 of the paper: forward pass, gradient of the loss
with respect to the output, backward pass through the transposed Jacobians
(Section 3.1), then kernel and bias gradients and the update (Section 3.2,
Algorithm 3).  Convolutions and max-filters call the nested-loop oracle; the
transfer function (bias, then half-wave rectification), the square loss
1/2 sum (out - target)^2 and the plain update p -= eta * g are written out in
numpy.  Readings the paper leaves open: the rectifier's derivative is 1 where
the forward output is > 0 and 0 elsewhere; the loss is not averaged; the
network input receives no backward image.
"""
from __future__ import annotations

import numpy as np

import oracle


def forward(layers, params, x):
    """Returns the list of node images: acts[0] = input, acts[l+1] = output of layer l.
    For max-filter layers the argmax offsets are kept in aux[l]."""
    acts = [np.asarray(x, dtype=np.float64)]
    aux = [None] * len(layers)
    for l, spec in enumerate(layers):
        a = acts[-1]
        if spec[0] == "conv":
            y = oracle.conv3d_fwd(a, params[l]["w"])
        elif spec[0] == "transfer":
            y = np.maximum(a + params[l]["b"][:, None, None, None], 0.0)
        elif spec[0] == "maxfilter":
            y, aux[l] = oracle.maxfilter3d_fwd(a, spec[1])
        else:
            raise ValueError(spec)
        acts.append(y)
    return acts, aux


def backward(layers, params, acts, aux, gout):
    """Gradients of the loss w.r.t. every parameter, given d loss / d output."""
    grads = [None] * len(layers)
    g = np.asarray(gout, dtype=np.float64)
    for l in range(len(layers) - 1, -1, -1):
        spec = layers[l]
        if spec[0] == "conv":
            grads[l] = {"w": oracle.conv3d_wgrad(acts[l], g)}
            g = oracle.conv3d_bwd(g, params[l]["w"], acts[l].shape[1:]) if l > 0 else None
        elif spec[0] == "transfer":
            g = g * (acts[l + 1] > 0.0)
            grads[l] = {"b": g.reshape(g.shape[0], -1).sum(axis=1)}
        elif spec[0] == "maxfilter":
            g = oracle.maxfilter3d_bwd(g, aux[l], acts[l].shape[1:], spec[1])
    return grads


def train_round(layers, params, x, target, eta):
    """One round; returns (loss, acts, aux, grads, updated params)."""
    acts, aux = forward(layers, params, x)
    diff = acts[-1] - np.asarray(target, dtype=np.float64)
    loss = 0.5 * float(np.sum(diff * diff))
    grads = backward(layers, params, acts, aux, diff)
    new = []
    for p, g in zip(params, grads):
        new.append(None if p is None else {k: np.asarray(v, dtype=np.float64) - eta * g[k] for k, v in p.items()})
    return loss, acts, aux, grads, new
