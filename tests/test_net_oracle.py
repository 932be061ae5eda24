"""Pins of the float64 network reference: its analytic gradients against central
differences of its own loss on a small net with the benchmark network's layer types."""
import numpy as np

from oracle import net as onet
from paper_1510_06706_amd import synth     # the seeded value generator only

import workloads

LAYERS = [("conv", 1, 3, (2, 2, 2)), ("transfer",), ("maxfilter", (2, 2, 1)),
          ("conv", 3, 2, (2, 1, 2)), ("transfer",)]
IN_SHAPE = (1, 6, 5, 6)


def loss_of(params, x, t):
    acts, _ = onet.forward(LAYERS, params, x)
    return 0.5 * float(np.sum((acts[-1] - t) ** 2))


def test_shapes_follow_the_valid_and_filter_size_rules():
    k3, m2 = (3, 3, 3), (2, 2, 2)
    config3 = [("conv", 1, 40, k3), ("transfer",), ("conv", 40, 40, k3), ("transfer",), ("maxfilter", m2),
               ("conv", 40, 40, k3), ("transfer",), ("conv", 40, 40, k3), ("transfer",), ("maxfilter", m2),
               ("conv", 40, 40, k3), ("transfer",), ("conv", 40, 3, k3), ("transfer",)]
    s = [a.shape for a in onet.forward(config3, workloads.layer_params(config3, 1), np.zeros((1, 26, 26, 26)))[0]]
    assert s[0] == (1, 26, 26, 26) and s[-1] == (3, 12, 12, 12)
    assert s[5] == (40, 21, 21, 21) and s[10] == (40, 16, 16, 16)


def test_analytic_gradients_match_finite_differences():
    params = workloads.layer_params(LAYERS, 5)
    for p in params:          # biases well away from the rectifier's kink for most voxels
        if p and "b" in p:
            p["b"] += 0.3
    x = synth.uniform_pm1(6, 0, IN_SHAPE).astype(np.float64)
    t = synth.uniform_01(6, 3, workloads.layer_shapes(LAYERS, IN_SHAPE)[-1]).astype(np.float64)
    loss, acts, aux, grads, new = onet.train_round(LAYERS, params, x, t, 1e-3)
    assert abs(loss - loss_of(params, x, t)) < 1e-12
    rs = np.random.RandomState(2)
    h = 1e-6
    checked = 0
    for l, p in enumerate(params):
        if p is None:
            continue
        for k, v in p.items():
            for _ in range(6):
                idx = tuple(rs.randint(0, s) for s in v.shape)
                old = v[idx]
                v[idx] = old + h; lp = loss_of(params, x, t)
                v[idx] = old - h; lm = loss_of(params, x, t)
                v[idx] = old
                fd = (lp - lm) / (2 * h)
                assert abs(fd - grads[l][k][idx]) < 1e-6 * max(1.0, abs(fd)), (l, k, idx, fd, grads[l][k][idx])
                checked += 1
            assert np.allclose(new[l][k], v - 1e-3 * grads[l][k], rtol=0, atol=1e-15)
    assert checked >= 24
