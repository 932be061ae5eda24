"""Float64 reference of one training round of a layered ConvNet (TEST INFRASTRUCTURE ONLY).

The round follows Section 3 of the paper: forward pass, gradient of the loss
with respect to the output, backward pass through the transposed Jacobians
(Section 3.1), then kernel and bias gradients and the update (Section 3.2,
Algorithm 3).  Convolutions, max-filters and max-pooling call the nested-loop
oracle; the transfer functions (bias, then nonlinearity), the losses and the
plain update p -= eta * g are written out in numpy.  Readings the paper leaves
open: the rectifier's derivative is 1 where the forward output is > 0 and 0
elsewhere; the loss is not averaged; the network input receives no backward
image.

Layer specs (tuples; trailing fields optional):
  ("conv", f, f', k[, s])      convolution layer, kernel extents k, sparsity s
  ("transfer"[, fn])           bias + "rectify" (default) | "logistic" | "tanh"
  ("maxfilter", win[, s])      sliding-window maximum, window taps s apart
  ("maxpool", p)               block maximum
"""
from __future__ import annotations

import numpy as np

import oracle


ONES = (1, 1, 1)


def _opt(spec, i, default):
    return spec[i] if len(spec) > i else default


def forward(layers, params, x):
    """Returns the list of node images: acts[0] = input, acts[l+1] = output of layer l.
    For max-filter layers the argmax offsets are kept in aux[l]."""
    acts = [np.asarray(x, dtype=np.float64)]
    aux = [None] * len(layers)
    for l, spec in enumerate(layers):
        a = acts[-1]
        if spec[0] == "conv":
            y = oracle.conv3d_fwd(a, params[l]["w"], _opt(spec, 4, ONES))
        elif spec[0] == "transfer":
            y = oracle.transfer_fwd(a, params[l]["b"], _opt(spec, 1, "rectify"))
        elif spec[0] == "maxfilter":
            y, aux[l] = oracle.maxfilter3d_fwd(a, spec[1], _opt(spec, 2, ONES))
        elif spec[0] == "maxpool":
            y, aux[l] = oracle.maxpool3d_fwd(a, spec[1])
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
            sp = _opt(spec, 4, ONES)
            grads[l] = {"w": oracle.conv3d_wgrad(acts[l], g, sp)}
            g = oracle.conv3d_bwd(g, params[l]["w"], acts[l].shape[1:], sp) if l > 0 else None
        elif spec[0] == "transfer":
            g = oracle.transfer_bwd(g, acts[l + 1], _opt(spec, 1, "rectify"))
            grads[l] = {"b": g.reshape(g.shape[0], -1).sum(axis=1)}
        elif spec[0] == "maxfilter":
            g = oracle.maxfilter3d_bwd(g, aux[l], acts[l].shape[1:], spec[1], _opt(spec, 2, ONES))
        elif spec[0] == "maxpool":
            g = oracle.maxpool3d_bwd(g, aux[l], acts[l].shape[1:], spec[1])
    return grads


def train_round(layers, params, x, target, eta, loss="square"):
    """One round; returns (loss value, acts, aux, grads, updated params)."""
    acts, aux = forward(layers, params, x)
    value = oracle.loss_value(acts[-1], target, loss)
    grads = backward(layers, params, acts, aux, oracle.loss_grad(acts[-1], target, loss))
    loss = value
    new = []
    for p, g in zip(params, grads):
        new.append(None if p is None else {k: np.asarray(v, dtype=np.float64) - eta * g[k] for k, v in p.items()})
    return loss, acts, aux, grads, new
