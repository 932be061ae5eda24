#!/usr/bin/env python3
"""Benchmark of the convolutional-layer hot path on one MI355X.

Workload: the wide 3D layer (fan-in 40 -> fan-out 40, 64^3 images, 5^3 kernels,
fp32, synthetic values).  One step trains the layer once with each method:

    direct : forward + backward + kernel gradient
    fft    : kernel spectra once, then forward + backward (streaming the resident
             spectra) + kernel gradient from the node spectra the two passes memoized
    plus the sliding max-filter forward/backward on a 40 x 22^3 node set.

`value` is output voxels per second: every step produces the layer's f'*n'^3
output voxels twice (once per method).  Per-method and per-pass times, the
roofline of the dominant kernel and the CPU oracle timed on a bounded sample
are reported in the same JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0


def cpu_baseline(cfg, inp, w, gout, budget_s=18.0):
    """The oracle as it stands, timed on sampled outputs of each pass, extrapolated to the layer."""
    import oracle
    rs = np.random.RandomState(1)
    fo_vox = cfg.out_voxels
    in_vox = cfg.fan_in * int(np.prod(cfg.image))
    gw_n = cfg.fan_in * cfg.fan_out * int(np.prod(cfg.kernel))
    macs_full = cfg.macs
    per = {"fwd": (fo_vox, lambda p: oracle.conv3d_fwd_at(inp, w, p)),
           "bwd": (in_vox, lambda p: oracle.conv3d_bwd_at(gout, w, cfg.image, p)),
           "wgrad": (gw_n, lambda p: oracle.conv3d_wgrad_at(inp, gout, p))}
    inp64, w64, g64 = (a.astype(np.float64) for a in (inp, w, gout))
    inp, w, gout = inp64, w64, g64
    est = {}
    samples = {}
    for name, (total, fn) in per.items():
        macs_each = macs_full / total
        n0 = max(16, int(2e8 / macs_each))
        pos = rs.randint(0, total, size=n0)
        t0 = time.perf_counter(); fn(pos); t1 = time.perf_counter()
        rate = n0 / max(t1 - t0, 1e-6)
        n1 = int(min(total, max(n0, rate * budget_s / 3.0)))
        pos = rs.randint(0, total, size=n1)
        t0 = time.perf_counter(); fn(pos); t1 = time.perf_counter()
        est[name] = (t1 - t0) * total / n1
        samples[name] = n1
    t_layer = est["fwd"] + est["bwd"] + est["wgrad"]
    return {"value": fo_vox / t_layer, "unit": "output voxels/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": "fp64 nested-loop oracle on %d fwd voxels, %d bwd voxels, %d kernel-gradient entries "
                      "drawn uniformly from the same layer, each a full-depth sum; layer time extrapolated "
                      "(fwd %.1f s, bwd %.1f s, wgrad %.1f s)" % (samples["fwd"], samples["bwd"], samples["wgrad"],
                                                                   est["fwd"], est["bwd"], est["wgrad"]),
            "gflops": 3 * 2 * macs_full / t_layer / 1e9}


def report_all_configs(path):
    """Per-pass times of every benchmark configuration (not part of the timed step): configs 1, 2, 4, 5 in
    both methods (config 5's FFT rows with resident kernel spectra), config 3 as a whole training round."""
    import torch
    from paper_1510_06706_amd import binding as znn
    from paper_1510_06706_amd import net as znet
    from paper_1510_06706_amd import synth

    def timed(fn, reps):
        fn(); fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / reps

    rows = []
    for cfg, modes in ((synth.CONFIG1, ("direct", "fft")), (synth.CONFIG2, ("direct", "fft")),
                       (synth.CONFIG4, ("direct", "fft")), (synth.CONFIG5, ("direct", "fft"))):
        inp, w, gout = synth.layer_tensors(cfg)
        d_in, d_w, d_g = (torch.from_numpy(a).to("cuda:0") for a in (inp, w, gout))
        del inp, w, gout
        for mode in modes:
            p = znn.Plan(cfg.fan_in, cfg.fan_out, cfg.image, cfg.kernel, mode)
            reps = 3 if cfg is synth.CONFIG5 else 10
            t = {}
            wk = d_w
            if mode == "fft":
                t["kernel_spectra"] = timed(lambda: p.prepare_kernels(d_w), reps)
                wk = None
            out = p.fwd(d_in, wk); gin = p.bwd(d_g, wk); gw = p.wgrad(d_in, d_g)
            t["fwd"] = timed(lambda: p.fwd(d_in, wk, out), reps)
            t["bwd"] = timed(lambda: p.bwd(d_g, wk, gin), reps)
            t["wgrad"] = timed(lambda: p.wgrad(d_in, d_g, gw), reps)
            tot = sum(t.values())
            rows.append({"config": cfg.name, "mode": mode, "ms": t, "layer_ms": tot,
                         "voxels_per_s": cfg.out_voxels / (tot * 1e-3),
                         "effective_tflops": 3 * 2.0 * cfg.macs / (tot * 1e-3) / 1e12})
            print("%-24s %-6s %s  layer %.3f ms  %.3g voxels/s  %.1f eff. TFLOP/s" %
                  (cfg.name, mode, " ".join("%s %.3f" % kv for kv in t.items()), tot, rows[-1]["voxels_per_s"],
                   rows[-1]["effective_tflops"]), file=sys.stderr, flush=True)
            p.close()
            del out, gin, gw
        del d_in, d_w, d_g
        torch.cuda.empty_cache()
    x, target, params = znet.config3_tensors()
    d_x, d_t = torch.from_numpy(x).to("cuda:0"), torch.from_numpy(target).to("cuda:0")
    for mode in ("direct", "fft"):
        net = znet.Net(znet.CONFIG3_LAYERS, znet.CONFIG3_INPUT, params, mode)
        ms = timed(lambda: net.train_round(d_x, d_t, znet.CONFIG3_ETA), 10)
        rows.append({"config": "c3_training_round", "mode": mode, "layer_ms": ms, "voxels_per_s": 3 * 12 ** 3 / (ms * 1e-3)})
        print("%-24s %-6s round %.3f ms  %.3g output voxels/s" % ("c3_training_round", mode, ms, rows[-1]["voxels_per_s"]),
              file=sys.stderr, flush=True)
    # whole rounds of the other networks: tuned strategies (direct / FFT / FFT with memoized
    # spectra per layer), the max-filtering net with sparse layers, the paper's 2D network
    for name, layers, in_shape, tensors in (
            ("c3_training_round", znet.CONFIG3_LAYERS, znet.CONFIG3_INPUT, (x, target, params)),
            ("c3_sparse_round", synth.CONFIG3_SPARSE_LAYERS, synth.CONFIG3_SPARSE_INPUT, synth.config3_sparse_tensors()),
            ("net2d_round", synth.CONFIG2D_LAYERS, synth.CONFIG2D_INPUT, synth.config2d_tensors())):
        xx, tt, pp = tensors
        d_x, d_t = torch.from_numpy(xx).to("cuda:0"), torch.from_numpy(tt).to("cuda:0")
        out_vox = int(np.prod(synth.shapes(layers, in_shape)[-1]))
        for mode in (("tuned",) if name == "c3_training_round" else ("direct", "fft", "tuned")):
            net = znet.Net(layers, in_shape, pp, mode)
            ms = timed(lambda: net.train_round(d_x, d_t, 1e-4), 10)
            row = {"config": name, "mode": mode, "layer_ms": ms, "voxels_per_s": out_vox / (ms * 1e-3)}
            if mode == "tuned":
                row["strategies"] = [net.strategy[l] for l in sorted(net.tuning)]
            rows.append(row)
            print("%-24s %-6s round %.3f ms  %.3g output voxels/s %s" % (name, mode, ms, row["voxels_per_s"],
                  row.get("strategies", "")), file=sys.stderr, flush=True)
            if mode == "tuned":     # the same round recorded once into a HIP graph and replayed
                replay, _ = net.capture_round(d_x, d_t, 1e-4)
                ms = timed(replay, 10)
                rows.append({"config": name, "mode": "tuned, HIP graph", "layer_ms": ms,
                             "voxels_per_s": out_vox / (ms * 1e-3)})
                print("%-24s %-6s round %.3f ms  %.3g output voxels/s (HIP graph replay)" %
                      (name, mode, ms, out_vox / (ms * 1e-3)), file=sys.stderr, flush=True)
            del net
        torch.cuda.empty_cache()
    # a multi-scale graph with converging branches, as a launch DAG on 1 and on 4 streams
    from paper_1510_06706_amd import graph as zgraph
    g = synth.multiscale_graph(width=40, n=40)
    inputs, targets, gp = synth.graph_tensors(g, 77)
    d_in = {n: torch.from_numpy(v).to("cuda:0") for n, v in inputs.items()}
    d_tg = {n: torch.from_numpy(v).to("cuda:0") for n, v in targets.items()}
    for streams in (1, 4):
        gn = zgraph.GraphNet(g, gp, "auto", streams=streams)
        ms = timed(lambda: gn.train_round(d_in, d_tg, 1e-4, "cross_entropy"), 10)
        rows.append({"config": "multiscale_graph_w40_n40", "mode": "auto, %d stream(s)" % streams, "layer_ms": ms})
        print("%-24s streams %d round %.3f ms" % ("multiscale_graph_w40_n40", streams, ms), file=sys.stderr, flush=True)
        del gn
    os.makedirs(os.path.dirname(path) or ".", exist_ok=True)
    with open(path, "w") as fh:
        json.dump(rows, fh, indent=1)
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for `rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE`: run two steps and a plain 1 GiB device "
                         "copy whose known size calibrates the counters, then exit")
    ap.add_argument("--direct-probe", action="store_true",
                    help="for `rocprofv3 --pmc <SQ counters>`: run the three direct-method passes of config 2 "
                         "three times and exit")
    ap.add_argument("--report-all", metavar="JSON", default=None,
                    help="also time every configuration pass by pass, print the table to stderr and write it here")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1510_06706_amd import binding as znn
    from paper_1510_06706_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    cfg = synth.CONFIG2
    inp, w, gout = synth.layer_tensors(cfg)
    d_in, d_w, d_g = (torch.from_numpy(a).to(dev) for a in (inp, w, gout))
    out = torch.empty((cfg.fan_out,) + cfg.out, dtype=torch.float32, device=dev)
    gin = torch.empty_like(d_in)
    gw = torch.empty_like(d_w)
    mf_n, mf_win = (22, 22, 22), (2, 2, 2)
    d_mf = torch.from_numpy(np.maximum(synth.uniform_pm1(1003, 0, (40,) + mf_n), 0)).to(dev)
    d_mfg = torch.from_numpy(synth.uniform_pm1(1003, 2, (40, 21, 21, 21))).to(dev)

    plans = {"direct": znn.Plan(cfg.fan_in, cfg.fan_out, cfg.image, cfg.kernel, "direct"),
             "fft": znn.Plan(cfg.fan_in, cfg.fan_out, cfg.image, cfg.kernel, "fft")}
    plans["fft"].enable_memo(dev)

    def run_mode(mode):
        p = plans[mode]
        if mode == "fft":       # the memoized schedule of Section 4: every spectrum is computed once
            p.prepare_kernels(d_w)
            p.fwd(d_in, None, out)
            p.bwd(d_g, None, gin)
            p.wgrad_memo(gw)
        else:
            p.fwd(d_in, d_w, out)
            p.bwd(d_g, d_w, gin)
            p.wgrad(d_in, d_g, gw)

    def step():
        run_mode("direct")
        run_mode("fft")
        _, idx = znn.maxfilter3d_fwd(d_mf, mf_win)
        znn.maxfilter3d_bwd(d_mfg, idx, mf_n, mf_win)

    if args.direct_probe:
        for _ in range(3):
            run_mode("direct")
        torch.cuda.synchronize()
        print(json.dumps({"direct_probe": "done", "launches_of_each_pass": 3}))
        return
    if args.traffic_probe:
        step(); step()
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        b = torch.empty_like(a)
        b.copy_(a)          # plain copy kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": "done", "copy_bytes_each_way": a.numel() * 4}))
        return

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # per-pass times with events on the stream the kernels run on (torch's current stream)
    def timed(fn, reps=10):
        fn(); fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / reps

    pd, pf = plans["direct"], plans["fft"]
    per = {"direct": {"fwd": timed(lambda: pd.fwd(d_in, d_w, out)),
                      "bwd": timed(lambda: pd.bwd(d_g, d_w, gin)),
                      "wgrad": timed(lambda: pd.wgrad(d_in, d_g, gw))}}
    t_ker = timed(lambda: pf.prepare_kernels(d_w))
    per["fft"] = {"kernel_spectra": t_ker,
                  "fwd": timed(lambda: pf.fwd(d_in, None, out)),
                  "bwd": timed(lambda: pf.bwd(d_g, None, gin)),
                  "wgrad": timed(lambda: pf.wgrad_memo(gw))}
    t_wgrad_alone = timed(lambda: pf.wgrad(d_in, d_g, gw))
    flop_pass = 2.0 * cfg.macs
    summary = {}
    for mode, t in per.items():
        tot = sum(t.values())
        summary[mode] = {"ms": {k: round(v, 4) for k, v in t.items()}, "layer_ms": round(tot, 4),
                         "voxels_per_s": cfg.out_voxels / (tot * 1e-3),
                         "effective_tflops": 3 * flop_pass / (tot * 1e-3) / 1e12}

    # per-kernel durations from HIP events recorded by the library around every launch,
    # on the stream the kernels run on; roofline of the kernel that dominates the step
    from paper_1510_06706_amd import roofline as rl
    trace_steps = 3
    torch.cuda.synchronize()
    znn.trace_enable(True)
    for _ in range(trace_steps):
        step()
    torch.cuda.synchronize()
    records = znn.trace_collect(65536)
    znn.trace_enable(False)
    roof, kernels = rl.report(cfg, plans["fft"].fft_extents, records, trace_steps)

    result = {
        "metric": "conv-layer fwd+bwd+wgrad output voxels/s (direct and FFT method, each once per step)",
        "value": 2 * cfg.out_voxels / (ms_per_step * 1e-3),
        "unit": "output voxels/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "wide 3D layer f=40 -> f'=40, n=64^3, k=5^3 (config 2), direct + FFT, "
                               "plus 2^3 max-filter on 40x22^3", "global_batch": 1},
        "effective_tflops_per_step": 2 * 3 * flop_pass / (ms_per_step * 1e-3) / 1e12,
        "per_mode": summary,
        "fft_wgrad_without_memo_ms": round(t_wgrad_alone, 4),
        "roofline": roof,
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, inp, w, gout)
    if args.report_all:
        del d_in, d_w, d_g, out, gin, gw
        for p in plans.values():
            p.close()
        torch.cuda.empty_cache()
        report_all_configs(args.report_all)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
