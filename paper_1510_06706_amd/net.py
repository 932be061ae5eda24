"""One training round of a layered ConvNet driven through the C ABI (config-3 harness).

This module only sequences library calls (Section 3 of the paper: forward pass,
loss gradient, backward pass, gradients, update); every arithmetic step runs in
libznn's kernels.  The layer lists of the benchmark networks and their seeded
synthetic tensors live in ``synth``.
"""
from __future__ import annotations

import numpy as np

from . import binding as znn
from .synth import ONES, _opt, shapes


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

    def capture_round(self, x, target, eta, loss="square"):
        """Records one training round (all library launches on the current HIP stream, no host
        synchronisation, no memset) into a HIP graph and returns ``(replay, outputs)``:
        ``replay()`` re-runs the round on the same buffers - new inputs are copied into ``x`` and
        ``target`` in place, the parameters are updated in place - without per-launch host cost;
        ``outputs = (acts, aux, gout, grads)`` are the graph's own output tensors.  Workspaces and
        resident spectra are allocated by a warm-up round before the capture."""
        import torch
        side = torch.cuda.Stream(device=self.device)
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):       # warm-up outside the graph: plans grow their workspaces
            saved = [None if p is None else {k: v.clone() for k, v in p.items()} for p in self.params]
            self.train_round(x, target, eta, loss=loss)
            for p, q in zip(self.params, saved):
                if p is not None:
                    for k in p:
                        p[k].copy_(q[k])
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            outputs = self.train_round(x, target, eta, loss=loss)
        return graph.replay, outputs
