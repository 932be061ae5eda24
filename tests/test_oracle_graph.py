"""Pins of the float64 graph reference (general computation graphs, Sections 2 and 3).

The sum at a convergent node is checked against scipy.signal convolutions of every
converging edge added up by hand; the backward pass (sum over outgoing edges, kernel and
bias gradients of every edge) against central differences of the graph's own loss; a
layered chain written as a graph against the layered reference.
"""
import numpy as np
import pytest
import scipy.signal

import oracle
from oracle import graph as ograph
from oracle import net as onet

import workloads


def f64(params):
    return {n: {k: v.astype(np.float64) for k, v in p.items()} for n, p in params.items()}


def small_graph():
    return workloads.multiscale_graph(width=2, n=11)


def test_convergent_node_is_the_sum_of_its_edges_computed_by_scipy():
    g = small_graph()
    inputs, targets, params = workloads.graph_tensors(g, 3)
    params = f64(params)
    img, aux = ograph.forward(g, params, inputs)
    a1, b1, m = img["a1"], img["b1"], img["m"]

    def stuffed(w, s):
        k = w.shape
        z = np.zeros(tuple(s[d] * (k[d] - 1) + 1 for d in range(3)))
        z[::s[0], ::s[1], ::s[2]] = w
        return z

    want = np.zeros_like(img["c"])
    for j in range(want.shape[0]):
        for src, name, s in ((b1, "c2", (1, 1, 1)), (a1, "c3", (2, 2, 2)), (m, "c4", (3, 3, 3))):
            for i in range(src.shape[0]):
                want[j] += scipy.signal.convolve(src[i], stuffed(params[name]["w"][j, i], s), mode="valid")
    np.testing.assert_allclose(img["c"], want, atol=1e-12)
    # the max-filter branch really filters
    assert np.array_equal(m, oracle.maxfilter3d_fwd(a1, (2, 2, 2))[0])


def test_graph_gradients_match_finite_differences_on_every_edge():
    g = small_graph()
    inputs, targets, params = workloads.graph_tensors(g, 4)
    params = f64(params)
    for p in params.values():
        if "b" in p:
            p["b"] += 0.3

    def loss_of():
        img, _ = ograph.forward(g, params, inputs)
        return sum(oracle.loss_value(img[n], targets[n], "cross_entropy") for n in g["outputs"])

    value, img, aux, grads, new = ograph.train_round(g, params, inputs, targets, 1e-3, "cross_entropy")
    assert abs(value - loss_of()) < 1e-12
    assert set(grads) == set(params)
    rs = np.random.RandomState(5)
    h = 1e-6
    for name, p in params.items():
        for k, v in p.items():
            for _ in range(5):
                q = tuple(rs.randint(0, s) for s in v.shape)
                old = v[q]
                v[q] = old + h; lp = loss_of()
                v[q] = old - h; lm = loss_of()
                v[q] = old
                fd = (lp - lm) / (2 * h)
                assert abs(fd - grads[name][k][q]) < 2e-6 * max(1.0, abs(fd)), (name, k, q, fd, grads[name][k][q])
            assert np.allclose(new[name][k], v - 1e-3 * grads[name][k], rtol=0, atol=1e-15)


def test_a_chain_written_as_a_graph_equals_the_layered_reference():
    layers = [("conv", 1, 3, (2, 2, 2)), ("transfer", "tanh"), ("maxfilter", (2, 1, 2)),
              ("conv", 3, 2, (2, 2, 1), (2, 1, 2)), ("transfer",), ("maxpool", (1, 2, 2)),
              ("conv", 2, 2, (1, 2, 1)), ("transfer", "logistic")]
    in_shape = (1, 8, 8, 8)
    x, t, lp = workloads.net_tensors(layers, in_shape, 12)
    lp = [None if p is None else {k: v.astype(np.float64) for k, v in p.items()} for p in lp]
    edges, params = [], {}
    for l, spec in enumerate(layers):
        name, src, dst = "e%d" % l, "n%d" % l, "n%d" % (l + 1)
        if spec[0] == "conv":
            edges.append(("conv", name, src, dst, spec[2]) + tuple(spec[3:]))
        else:
            edges.append((spec[0], name, src, dst) + tuple(spec[1:]))
        if lp[l] is not None:
            params[name] = lp[l]
    g = {"inputs": {"n0": in_shape}, "edges": edges, "outputs": ["n%d" % len(layers)]}
    assert workloads.graph_shapes(g)["n%d" % len(layers)] == workloads.layer_shapes(layers, in_shape)[-1]
    v1, acts, _, g1, _ = onet.train_round(layers, lp, x, t, 1e-2, "cross_entropy")
    v2, img, _, g2, _ = ograph.train_round(g, params, {"n0": x}, {"n%d" % len(layers): t}, 1e-2, "cross_entropy")
    assert v1 == v2
    for l in range(len(layers)):
        assert np.array_equal(acts[l + 1], img["n%d" % (l + 1)])
        if g1[l] is not None:
            for k in g1[l]:
                assert np.array_equal(g1[l][k], g2["e%d" % l][k])


def test_order_rejects_unreachable_sources():
    g = {"inputs": {"x": (1, 4, 4, 4)}, "edges": [("transfer", "t", "nowhere", "y")], "outputs": ["y"]}
    with pytest.raises(ValueError):
        ograph.order(g)
