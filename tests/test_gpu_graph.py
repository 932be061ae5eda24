"""Parity of the multi-stream graph executor with the float64 graph reference, and the
paper's 2D benchmark network as a second end-to-end workload."""
import numpy as np
import pytest

from oracle import graph as ograph
from oracle import net as onet
from paper_1510_06706_amd import binding as znn
from paper_1510_06706_amd import graph as zgraph
from paper_1510_06706_amd import net as znet
from paper_1510_06706_amd import synth

pytestmark = pytest.mark.gpu

TOL = {"direct": 1e-4, "fft": 1e-3}


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def host(t):
    import torch
    torch.cuda.synchronize()
    return t.cpu().numpy()


def rel_err(got, ref):
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - ref)) / max(np.max(np.abs(ref)), 1e-300))


@pytest.mark.parametrize("mode", ["direct", "fft"])
def test_multiscale_graph_round_matches_the_reference(mode):
    import torch
    g = synth.multiscale_graph()
    inputs, targets, params = synth.graph_tensors(g, 51)
    p64 = {n: {k: v.astype(np.float64) for k, v in p.items()} for n, p in params.items()}
    value, r_img, r_aux, r_grads, r_new = ograph.train_round(g, p64, inputs, targets, 0.05, "cross_entropy")
    results = []
    for streams in (4, 1):
        net = zgraph.GraphNet(g, params, mode, streams=streams)
        img, aux, gout, grads = net.train_round({n: dev(v) for n, v in inputs.items()},
                                                {n: dev(v) for n, v in targets.items()}, 0.05, "cross_entropy")
        torch.cuda.synchronize()
        for n in r_img:
            assert rel_err(host(img[n]), r_img[n]) <= TOL[mode], ("image", n)
        assert np.array_equal(host(aux["m0"]), r_aux["m0"])
        for name, gr in r_grads.items():
            for k in gr:
                assert rel_err(host(grads[name][k]), gr[k]) <= TOL[mode], ("gradient", name, k)
                assert rel_err(host(net.params[name][k]), r_new[name][k]) <= TOL[mode], ("update", name, k)
        results.append({(name, k): host(v) for name, gr in grads.items() for k, v in gr.items()})
    # the number of streams changes the schedule, not one bit of the result
    for key in results[0]:
        assert np.array_equal(results[0][key], results[1][key]), key


def test_graph_rejects_a_node_that_reaches_no_output():
    g = synth.multiscale_graph()
    g["outputs"] = ["y"]
    with pytest.raises(ValueError):
        zgraph.GraphNet(g, synth.graph_params(g, 1), "direct")


@pytest.mark.timeout(600)
@pytest.mark.parametrize("mode", ["fft", "auto"])
def test_two_dimensional_benchmark_network_round(mode):
    """Six 11x11 convolutional layers, 48x48 output patch (Section 6): the FFT method is
    the one the paper uses in 2D; 'auto' takes the library's own choice per layer."""
    import torch
    layers, in_shape = synth.CONFIG2D_LAYERS, synth.CONFIG2D_INPUT
    x, target, params = synth.config2d_tensors()
    net = znet.Net(layers, in_shape, params, mode)
    acts, aux, gout, grads = net.train_round(dev(x), dev(target), 1e-4)
    torch.cuda.synchronize()
    p64 = [None if p is None else {k: v.astype(np.float64) for k, v in p.items()} for p in params]
    r_acts, r_aux = onet.forward(layers, p64, x)
    assert rel_err(host(acts[-1]), r_acts[-1]) <= 1e-3
    # the backward pass of the reference takes the GPU's argmax and rectifier decisions where
    # they differ (near-ties, checked), as in the 3D network test
    sel_aux, sel_acts = list(r_aux), list(r_acts)
    for l, spec in enumerate(layers):
        if spec[0] == "maxfilter":
            g_idx = host(aux[l])
            bad = g_idx != r_aux[l]
            if bad.any():
                picked = np.take_along_axis(r_acts[l].reshape(r_acts[l].shape[0], -1),
                                            g_idx.reshape(g_idx.shape[0], -1).astype(np.int64), axis=1).reshape(g_idx.shape)
                assert np.max(np.abs(picked - r_acts[l + 1])[bad]) <= 1e-5 * np.max(np.abs(r_acts[l]))
                sel_aux[l] = g_idx
        elif spec[0] == "transfer":
            g_y = host(acts[l + 1])
            bad = (g_y > 0) != (r_acts[l + 1] > 0)
            if bad.any():
                pre = r_acts[l] + p64[l]["b"][:, None, None, None]
                assert np.max(np.abs(pre[bad])) <= 1e-5 * np.max(np.abs(pre))
                fixed = r_acts[l + 1].copy()
                fixed[bad] = g_y[bad]
                sel_acts[l + 1] = fixed
    r_grads = onet.backward(layers, p64, sel_acts, sel_aux, r_acts[-1] - target.astype(np.float64))
    worst = 0.0
    for l, g in enumerate(r_grads):
        if g is not None:
            for k in g:
                worst = max(worst, rel_err(host(grads[l][k]), g[k]))
    print("2D net %s: modes %s worst gradient rel-err %.2e" % (mode, [m for m in net.modes() if m is not None], worst),
          flush=True)
    assert worst <= 1e-3


def test_captured_training_round_replays_bit_for_bit():
    """A round recorded into a HIP graph gives, replay after replay and with eager work in
    between, exactly the parameters of the same number of eager rounds (the kernels are
    deterministic, the graph holds no memset nodes)."""
    import torch
    layers = [("conv", 2, 6, (3, 3, 3)), ("transfer",), ("maxfilter", (2, 2, 2)),
              ("conv", 6, 5, (2, 3, 2), (2, 2, 2)), ("transfer", "tanh"),
              ("conv", 5, 3, (3, 1, 2)), ("transfer", "logistic")]
    in_shape = (2, 14, 15, 16)
    x, target, params = synth.net_tensors(layers, in_shape, 61)
    for mode in ("direct", "fft"):
        eager = znet.Net(layers, in_shape, params, mode)
        graphed = znet.Net(layers, in_shape, params, mode)
        d_x, d_t = dev(x), dev(target)
        g_x, g_t = dev(x), dev(target)
        replay, outputs = graphed.capture_round(g_x, g_t, 0.05)
        for rnd in range(4):
            xr = synth.uniform_pm1(70 + rnd, 0, in_shape)         # new input every round
            d_x.copy_(dev(xr)); g_x.copy_(dev(xr))
            e_acts, _, _, e_grads = eager.train_round(d_x, d_t, 0.05)
            replay()
            torch.cuda.synchronize()
            assert np.array_equal(host(outputs[0][-1]), host(e_acts[-1])), (mode, rnd, "output")
            for l, p in enumerate(eager.params):
                if p is not None:
                    for k in p:
                        assert np.array_equal(host(graphed.params[l][k]), host(p[k])), (mode, rnd, l, k)
            # unrelated eager work between replays
            scratch = znn.transfer_fwd(d_x, dev(np.zeros(in_shape[0], dtype=np.float32)))
            del scratch
