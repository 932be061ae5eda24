"""One training round on a general computation graph, run as a multi-stream launch DAG.

Section 2 of the paper: nodes hold images, edges are convolutions, max-filters, max-pools
or transfer functions, and a node's image is the sum of the edges converging on it; the
graph need not be layered (branches with different sparsity may fan out of a node and
converge again: multi-scale nets).  Section 3: the backward graph is the same graph
reversed, a node's backward image being the sum over its outgoing edges.

The paper's CPU design runs the edges as tasks on worker threads.  On the GPU the same
dependency structure becomes streams and events: every edge is launched on one of a few
HIP streams after waiting for the event of its source node, so independent branches
overlap on the device, and the kernel-gradient of an edge runs on another stream than
its backward image (they only share inputs).  Sums at nodes are taken in the fixed order
of the edge list (every converging edge writes its own buffer, then the buffers are added
one by one), so results do not depend on which stream finished first.  Every tensor of a
round stays referenced until the round has joined the calling stream, and the next round
starts from events recorded after that join, so memory handed back to the allocator is never
reused while another stream still reads it.

This module only sequences library calls; every arithmetic step runs in libznn's kernels.
The graph format is the one of ``synth.graph_shapes``.
"""
from __future__ import annotations

import numpy as np

from . import binding as znn
from .synth import ONES, _opt, graph_shapes


def edge_order(graph):
    """Edge list reordered so that all edges into a node precede every edge out of it."""
    edges = list(graph["edges"])
    remaining_in = {}
    for e in edges:
        remaining_in[e[3]] = remaining_in.get(e[3], 0) + 1
    ready = set(graph["inputs"])
    out, pending = [], edges
    while pending:
        rest = []
        for e in pending:
            if e[2] in ready:
                out.append(e)
                remaining_in[e[3]] -= 1
                if remaining_in[e[3]] == 0:
                    ready.add(e[3])
            else:
                rest.append(e)
        if len(rest) == len(pending):
            raise ValueError("graph has a cycle or an edge whose source is never produced")
        pending = rest
    return out


class GraphNet:
    """Device-side state of a computation graph: plans per convolution edge, parameters as
    CUDA tensors, a pool of HIP streams (all at the default priority).

    Rounds run eagerly only.  Recording a round into a HIP graph is deliberately not offered:
    this executor waits on pooled events that were created and first recorded outside any
    capture, and joins its side streams (among them the kernel-gradient stream) to the
    calling stream only through the events of later edges, so a capture would contain waits on
    uncaptured work and forked streams that are never joined back before the capture ends;
    recording it that way crashed inside the runtime's end-of-capture call.  A capturable
    executor needs events created inside the capture, every side stream forked from the
    capturing stream, and a join of every side stream before the capture ends.  Layered nets
    (``net.Net.capture_round``) run on one stream and can be recorded."""

    def __init__(self, graph, params, mode="auto", device="cuda:0", streams=4):
        import torch
        self.graph = graph
        self.device = device
        self.shapes = graph_shapes(graph)
        self.edges = edge_order(graph)
        self.params = {n: {k: torch.from_numpy(np.ascontiguousarray(v)).to(device) for k, v in p.items()}
                       for n, p in params.items()}
        self.streams = [torch.cuda.Stream(device=device) for _ in range(max(1, int(streams)))]
        self._events, self._next_event = [], 0      # events are reused from round to round
        self.incoming, self.outgoing = {}, {}
        for e in self.edges:
            self.incoming.setdefault(e[3], []).append(e[1])
            self.outgoing.setdefault(e[2], []).append(e[1])
        for n in self.shapes:
            if n not in graph["outputs"] and n not in self.outgoing:
                raise ValueError("node %r reaches no output" % (n,))
        # two plans per convolution edge: forward/backward image on one stream, kernel gradient
        # on another, each with its own workspace
        self.plans, self.plans_w = {}, {}
        for e in self.edges:
            if e[0] == "conv":
                f, n = self.shapes[e[2]][0], self.shapes[e[2]][1:]
                m = mode[e[1]] if isinstance(mode, dict) else mode
                self.plans[e[1]] = znn.Plan(f, e[4], n, e[5], m, _opt(e, 6, ONES))
                self.plans_w[e[1]] = znn.Plan(f, e[4], n, e[5], self.plans[e[1]].mode, _opt(e, 6, ONES))

    def modes(self):
        return {n: p.mode for n, p in self.plans.items()}

    # ------------------------------------------------------------ helpers
    def _stream_of(self, i):
        return self.streams[i % len(self.streams)]

    def _event(self, stream):
        """An event from the pool, recorded on `stream`."""
        import torch
        if self._next_event == len(self._events):
            self._events.append(torch.cuda.Event())
        ev = self._events[self._next_event]
        self._next_event += 1
        ev.record(stream)
        return ev

    @staticmethod
    def _sum_in_order(parts, order, events, stream):
        """parts[name] are separate buffers; adds them in `order` on `stream` after their events."""
        import torch
        for name in order:
            stream.wait_event(events[name])
        total = parts[order[0]]
        if len(order) > 1:
            with torch.cuda.stream(stream):
                total = total.clone()   # the first part stays intact (it may be an edge's kept output)
        for name in order[1:]:
            znn.accumulate(total, parts[name], stream=stream)
        return total

    # ------------------------------------------------------------ passes
    def forward(self, inputs):
        """inputs: {node: CUDA tensor}.  Returns (node images, per-edge aux, node events)."""
        import torch
        main = torch.cuda.current_stream()
        self._next_event = 0
        img, aux, ready = dict(inputs), {}, {}
        first = self._event(main)
        for n in inputs:
            ready[n] = first
        parts, part_ev = {}, {}
        for i, e in enumerate(self.edges):
            kind, name, src, dst = e[:4]
            s = self._stream_of(i)
            s.wait_event(ready[src])
            a = img[src]
            if kind == "conv":
                y = self.plans[name].fwd(a, self.params[name]["w"], stream=s)
            elif kind == "transfer":
                y = aux[name] = znn.transfer_fwd(a, self.params[name]["b"], _opt(e, 4, "rectify"), stream=s)
            elif kind == "maxfilter":
                y, aux[name] = znn.maxfilter3d_fwd(a, e[4], _opt(e, 5, ONES), stream=s)
            else:
                y, aux[name] = znn.maxpool3d_fwd(a, e[4], stream=s)
            parts.setdefault(dst, {})[name] = y
            part_ev[name] = self._event(s)
            if len(parts[dst]) == len(self.incoming[dst]):       # last edge into dst: take the sum
                img[dst] = self._sum_in_order(parts[dst], self.incoming[dst], part_ev, s)
                ready[dst] = part_ev[name] if len(self.incoming[dst]) == 1 else self._event(s)
        for n in self.graph["outputs"]:
            main.wait_event(ready[n])
        return img, aux, ready

    def backward(self, img, aux, gout):
        """gout: {output node: d loss / d image} (valid on the current stream).  Returns
        (parameter gradients per edge name, backward images per node)."""
        import torch
        main = torch.cuda.current_stream()
        back, ready, grads, grad_ev = {}, {}, {}, []
        parts, part_ev = {}, {}
        start = self._event(main)     # forward images and gout are complete at this point of `main`
        for n, g in gout.items():
            parts.setdefault(n, {})["loss"] = g
            part_ev["loss:" + n] = start

        def finish(node, stream):
            order = ["loss"] * (node in gout) + list(reversed(self.outgoing.get(node, [])))
            evs = {k: part_ev["loss:" + node] if k == "loss" else part_ev[k] for k in order}
            back[node] = self._sum_in_order(parts[node], order, evs, stream)
            ready[node] = self._event(stream)

        for n in gout:
            if n not in self.outgoing:
                finish(n, main)
        for i, e in enumerate(reversed(self.edges)):
            kind, name, src, dst = e[:4]
            s = self._stream_of(i)
            s.wait_event(ready[dst])
            s.wait_event(start)
            g = back[dst]
            if kind == "conv":
                sw = self._stream_of(i + 1 + len(self.streams) // 2)
                sw.wait_event(ready[dst])
                sw.wait_event(start)
                grads[name] = {"w": self.plans_w[name].wgrad(img[src], g, stream=sw)}
                grad_ev.append(self._event(sw))
                gs = None if src in self.graph["inputs"] else self.plans[name].bwd(g, self.params[name]["w"], stream=s)
            elif kind == "transfer":
                gs = znn.transfer_bwd(g, aux[name], _opt(e, 4, "rectify"), stream=s)
                grads[name] = {"b": znn.bias_grad(gs, stream=s)}
            elif kind == "maxfilter":
                gs = znn.maxfilter3d_bwd(g, aux[name], self.shapes[src][1:], e[4], _opt(e, 5, ONES), stream=s)
            else:
                gs = znn.maxpool3d_bwd(g, aux[name], self.shapes[src][1:], e[4], stream=s)
            ev = self._event(s)
            grad_ev.append(ev)
            if gs is None:
                continue
            parts.setdefault(src, {})[name] = gs
            part_ev[name] = ev
            if len(parts[src]) == len(self.outgoing[src]) + (src in gout):
                finish(src, s)
        for ev in grad_ev:
            main.wait_event(ev)
        return grads, back

    def train_round(self, inputs, targets, eta, loss="square"):
        """Forward, loss gradient at every output node, backward, update (Algorithm 3).  The
        update runs after every stream has joined: kernels are read by the backward edges."""
        img, aux, _ = self.forward(inputs)
        gout = {n: znn.loss_grad(img[n], targets[n], loss) for n in self.graph["outputs"]}
        grads, back = self.backward(img, aux, gout)
        for name, p in self.params.items():
            for k in p:
                znn.sgd_update(p[k], grads[name][k], eta)
        return img, aux, gout, grads
