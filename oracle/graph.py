"""Float64 reference of one training round on a general computation graph
(TEST INFRASTRUCTURE ONLY).

Section 2 of the paper ("Computation graph"): nodes hold images, edges are the four
operations (convolution, max-pooling, max-filtering, transfer function); a node's image
is the sum of the outputs of the edges converging on it.  Section 3.1: the backward graph
is the same graph with every edge reversed and replaced by its transposed Jacobian, so a
node's backward image is the sum over its outgoing edges; output nodes start from the
gradient of the loss.  Section 3.2: kernel gradient from the forward image at the edge's
source and the backward image at its target; bias gradient as the sum of the backward
image after the transfer function's derivative.  The graph need not be layered: nodes
may fan out into branches with different sparsity (multi-scale) that converge again.

Here a "node" is a group of f images of equal extents and an "edge" is the whole bundle
of operations between two groups (f*f' convolutions, or f filters), the unit the GPU
library also works in.

Edges (tuples; ``name`` keys the edge's parameters):
  ("conv", name, src, dst, f_out, k[, s])     params {"w": [f_out, f_src, kz, ky, kx]}
  ("transfer", name, src, dst[, fn])           params {"b": [f]}
  ("maxfilter", name, src, dst, win[, s])
  ("maxpool", name, src, dst, p)
The graph is {"inputs": {node: shape}, "edges": [...], "outputs": [node, ...]}; every
edge's source must be complete before the edge runs, so edges are visited in an order
in which each node's incoming edges all precede its outgoing ones (checked).
"""
from __future__ import annotations

import numpy as np

import oracle

ONES = (1, 1, 1)


def _opt(e, i, default):
    return e[i] if len(e) > i else default


def order(graph):
    """Edges sorted so that all edges into a node come before any edge out of it."""
    edges = list(graph["edges"])
    incoming = {}
    for e in edges:
        incoming.setdefault(e[3], []).append(e[1])
    done_nodes = set(graph["inputs"])
    done_edges, out = set(), []
    while len(out) < len(edges):
        progressed = False
        for e in edges:
            if e[1] in done_edges or e[2] not in done_nodes:
                continue
            out.append(e)
            done_edges.add(e[1])
            progressed = True
            if all(n in done_edges for n in incoming[e[3]]):
                done_nodes.add(e[3])
        if not progressed:
            raise ValueError("graph has a cycle or an edge whose source is never produced")
    return out


def forward(graph, params, inputs):
    """Returns (node images, per-edge auxiliaries: argmax offsets of filters and pools, the
    own output of every transfer edge)."""
    img = {n: np.asarray(v, dtype=np.float64) for n, v in inputs.items()}
    aux = {}
    for e in order(graph):
        kind, name, src, dst = e[:4]
        a = img[src]
        if kind == "conv":
            y = oracle.conv3d_fwd(a, params[name]["w"], _opt(e, 6, ONES))
        elif kind == "transfer":
            y = aux[name] = oracle.transfer_fwd(a, params[name]["b"], _opt(e, 4, "rectify"))
        elif kind == "maxfilter":
            y, aux[name] = oracle.maxfilter3d_fwd(a, e[4], _opt(e, 5, ONES))
        elif kind == "maxpool":
            y, aux[name] = oracle.maxpool3d_fwd(a, e[4])
        else:
            raise ValueError(e)
        img[dst] = y if dst not in img else img[dst] + y
    return img, aux


def backward(graph, params, img, aux, gout):
    """``gout`` maps every output node to d loss / d image.  Returns (parameter gradients
    per edge name, backward images per node)."""
    back = {n: np.asarray(g, dtype=np.float64) for n, g in gout.items()}
    grads = {}
    for e in reversed(order(graph)):
        kind, name, src, dst = e[:4]
        if dst not in back:
            raise ValueError("node %r reaches no output" % (dst,))
        g = back[dst]
        if kind == "conv":
            sp = _opt(e, 6, ONES)
            grads[name] = {"w": oracle.conv3d_wgrad(img[src], g, sp)}
            gs = oracle.conv3d_bwd(g, params[name]["w"], img[src].shape[1:], sp)
        elif kind == "transfer":
            gs = oracle.transfer_bwd(g, aux[name], _opt(e, 4, "rectify"))      # aux: this edge's own output
            grads[name] = {"b": gs.reshape(gs.shape[0], -1).sum(axis=1)}
        elif kind == "maxfilter":
            gs = oracle.maxfilter3d_bwd(g, aux[name], img[src].shape[1:], e[4], _opt(e, 5, ONES))
        else:
            gs = oracle.maxpool3d_bwd(g, aux[name], img[src].shape[1:], e[4])
        back[src] = gs if src not in back else back[src] + gs
    return grads, back


def train_round(graph, params, inputs, targets, eta, loss="square"):
    """One round; the loss is summed over the output nodes.  Returns
    (loss value, node images, aux, gradients, updated params)."""
    img, aux = forward(graph, params, inputs)
    value = sum(oracle.loss_value(img[n], targets[n], loss) for n in graph["outputs"])
    gout = {n: oracle.loss_grad(img[n], targets[n], loss) for n in graph["outputs"]}
    grads, _ = backward(graph, params, img, aux, gout)
    new = {name: {k: np.asarray(v, dtype=np.float64) - eta * grads[name][k] for k, v in p.items()}
           for name, p in params.items()}
    return value, img, aux, grads, new
