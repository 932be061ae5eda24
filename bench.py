#!/usr/bin/env python3
"""Benchmark of the convolutional-layer hot path on one MI355X.

Headline workload: the largest of the five benchmark configurations, config 5 (fan-in 120 ->
fan-out 120, 96^3 images, 7^3 kernels, fp32, synthetic values).  One step trains that layer once
with the method the per-layer autotuner picks for it (Section 4): for the FFT method that is the
kernel transforms (once per step: the update changes the kernels), the forward and the backward
pass streaming the resident kernel spectra, and the kernel gradient from the node spectra the two
passes memoized; for the direct method the three passes.  `value` = f' n'^3 / t_step output voxels
per second.  The same JSON line carries, under `configs`, every pass of every configuration in both
methods with the roofline of each of its steps (configs 1, 2, 4, 5; config 5 also with the kernel
spectra kept in full, 52 GB; config 3 as whole training rounds; the max-filter pair), the roofline
of the kernel that dominates the headline step, and the CPU oracle timed on a sample of config 5.
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

TRAFFIC_PROFILE = "profiles/config5_hbm_traffic_pmc.txt"


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def cpu_baseline(cfg, inp, w, gout, budget_s=18.0, floor=(4096, 4096, 1024)):
    """The oracle as it stands, timed on sampled outputs of each pass, extrapolated to the layer."""
    import oracle
    rs = np.random.RandomState(1)
    fo_vox = cfg.out_voxels
    in_vox = cfg.fan_in * int(np.prod(cfg.image))
    gw_n = cfg.fan_in * cfg.fan_out * int(np.prod(cfg.kernel))
    macs_full = cfg.macs
    inp, w, gout = (a.astype(np.float64) for a in (inp, w, gout))
    per = {"fwd": (fo_vox, floor[0], lambda p: oracle.conv3d_fwd_at(inp, w, p)),
           "bwd": (in_vox, floor[1], lambda p: oracle.conv3d_bwd_at(gout, w, cfg.image, p)),
           "wgrad": (gw_n, floor[2], lambda p: oracle.conv3d_wgrad_at(inp, gout, p))}
    est, samples = {}, {}
    for name, (total, least, fn) in per.items():
        macs_each = macs_full / total
        n0 = max(16, int(2e8 / macs_each))
        pos = rs.randint(0, total, size=n0)
        t0 = time.perf_counter(); fn(pos); t1 = time.perf_counter()
        rate = n0 / max(t1 - t0, 1e-6)
        n1 = int(min(total, max(n0, least, rate * budget_s / 3.0)))
        pos = rs.randint(0, total, size=n1)
        t0 = time.perf_counter(); fn(pos); t1 = time.perf_counter()
        est[name] = (t1 - t0) * total / n1
        samples[name] = n1
    t_layer = est["fwd"] + est["bwd"] + est["wgrad"]
    return {"value": fo_vox / t_layer, "unit": "output voxels/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": "sampled: fp64 nested-loop oracle on %d forward voxels, %d backward voxels, %d kernel-gradient "
                      "entries drawn uniformly from the %s layer, each a full-depth sum; layer time extrapolated "
                      "(fwd %.0f s, bwd %.0f s, wgrad %.0f s)" % (samples["fwd"], samples["bwd"], samples["wgrad"],
                                                                   cfg.name, est["fwd"], est["bwd"], est["wgrad"]),
            "gflops": 3 * 2 * macs_full / t_layer / 1e9}


class Timer:
    """The paper's protocol (warm-up rounds, then the mean of the timed ones) with HIP events on the
    stream the kernels are launched on, and the library's own per-launch events for the step table."""

    def __init__(self, warmup, steps, cap_s=1.5):
        self.warmup, self.steps, self.cap_s = warmup, steps, cap_s

    def run(self, fn):
        import torch
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter(); fn(); torch.cuda.synchronize()
        once = max(time.perf_counter() - t0, 1e-5)
        reps = int(max(3, min(self.steps, self.cap_s / once)))
        for _ in range(max(0, min(self.warmup, reps) - 2)):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / reps, reps

    def trace(self, fn, reps=3):
        import torch
        from paper_1510_06706_amd import binding as znn
        torch.cuda.synchronize()
        znn.trace_enable(True)
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        rec = znn.trace_collect(65536)
        znn.trace_enable(False)
        return rec, reps


def pass_rows(timer, cfg, label, mode, layout, plan, d_in, d_w, d_g, bufs, resident, memo, meaningful=True):
    """One row per pass of a layer in one method: ms, voxels/s, effective TFLOP/s, and the roofline of every
    step of the pass (the pass row itself carries the figures of its slowest priced step)."""
    from paper_1510_06706_amd import roofline as rl
    out, gin, gw = bufs
    N = plan.fft_extents
    wk = None if resident else d_w
    calls = []
    if mode == "fft" and resident:
        calls.append(("kernel_spectra", lambda: plan.prepare_kernels(d_w)))
    calls += [("fwd", lambda: plan.fwd(d_in, wk, out)), ("bwd", lambda: plan.bwd(d_g, wk, gin))]
    if mode == "fft" and memo:
        calls.append(("wgrad_memo", lambda: plan.wgrad_memo(gw)))
    calls.append(("wgrad", lambda: plan.wgrad(d_in, d_g, gw)))
    rows = []
    for what, fn in calls:
        ms, reps = timer.run(fn)
        rec, treps = timer.trace(fn, 2 if ms > 50 else 3)
        steps = rl.steps_of_pass(rec, treps, cfg, N, layout, what)
        row = {"config": label, "layer": cfg.name, "mode": mode, "pass": what, "ms": ms, "timed_reps": reps}
        if mode == "fft":
            row["kernel_spectra"] = layout + (", resident" if resident else ", transformed inside the pass")
        if what != "kernel_spectra":
            row["voxels_per_s"] = cfg.out_voxels / (ms * 1e-3)
            row["effective_tflops"] = 2.0 * cfg.macs / (ms * 1e-3) / 1e12
        dom = rl.dominant(steps)
        if dom is not None:
            row["dominant_step"] = dom["step"]
            for k in ("bound", "achieved", "peak", "unit", "frac", "frac_of_unpacked_peak"):
                if k in dom:
                    row[k] = dom[k]
            if not meaningful:
                row["frac_note"] = "not meaningful: the layer is bound by launch latency, read the absolute time"
        row["steps"] = [{k: (round(v, 5) if isinstance(v, float) else v) for k, v in s.items()} for s in steps]
        rows.append(row)
        log("%-3s %-6s %-14s %9.4f ms  %s" % (label, mode, what, ms,
            "" if dom is None else "%s %.4g %s = %.3f of peak" % (dom["step"], dom["achieved"], dom["unit"], dom["frac"])))
    return rows


def layer_rows(timer, cfg, label, variants, meaningful=True):
    """All passes of one layer shape in the listed (mode, layout, resident, memo) variants."""
    import torch
    from paper_1510_06706_amd import binding as znn
    from paper_1510_06706_amd import synth
    dev = torch.device("cuda:0")
    inp, w, gout = synth.layer_tensors(cfg)
    d_in, d_w, d_g = (torch.from_numpy(a).to(dev) for a in (inp, w, gout))
    bufs = (torch.empty((cfg.fan_out,) + cfg.out, dtype=torch.float32, device=dev), torch.empty_like(d_in),
            torch.empty_like(d_w))
    rows = []
    for mode, layout, resident, memo in variants:
        p = znn.Plan(cfg.fan_in, cfg.fan_out, cfg.image, cfg.kernel, mode)
        if mode == "fft":
            if layout is not None:
                p.set_spectra_layout(layout)
            layout = p.spectra_layout
            if memo:
                p.enable_memo(dev)
        rows += pass_rows(timer, cfg, label, mode, layout, p, d_in, d_w, d_g, bufs, resident, memo, meaningful)
        p.close()
        del p
        torch.cuda.empty_cache()
    return rows, (inp, w, gout), (d_in, d_w, d_g), bufs


def config3_rows(timer):
    """Config 3 (a whole training round of the six-layer net) per method, and its two max-filters alone."""
    import torch
    from paper_1510_06706_amd import binding as znn
    from paper_1510_06706_amd import net as znet
    from paper_1510_06706_amd import roofline as rl
    from paper_1510_06706_amd import synth
    rows = []
    x, target, params = synth.config3_tensors()
    d_x, d_t = torch.from_numpy(x).to("cuda:0"), torch.from_numpy(target).to("cuda:0")
    out_vox = 3 * 12 ** 3
    for mode in ("direct", "fft", "tuned"):
        net = znet.Net(synth.CONFIG3_LAYERS, synth.CONFIG3_INPUT, params, mode)
        ms, reps = timer.run(lambda: net.train_round(d_x, d_t, synth.CONFIG3_ETA))
        row = {"config": "C3", "layer": "training round: 6 conv layers 3^3 of width 40, 26^3 -> 12^3, rectifiers, two 2^3 max-filters",
               "mode": mode, "pass": "forward + backward + update", "ms": ms, "timed_reps": reps,
               "voxels_per_s": out_vox / (ms * 1e-3),
               "frac_note": "not meaningful: ~80 small launches, bound by launch latency; read the absolute time"}
        if mode == "tuned":
            row["strategies"] = [net.strategy[l] for l in sorted(net.tuning)]
            replay, _ = net.capture_round(d_x, d_t, synth.CONFIG3_ETA)
            gms, greps = timer.run(replay)
            rows.append(dict(row, mode="tuned, replayed from a HIP graph", ms=gms, timed_reps=greps,
                             voxels_per_s=out_vox / (gms * 1e-3)))
        rows.append(row)
        log("C3  %-6s round %.4f ms" % (mode, ms))
        del net
    for maps, n, win in ((40, (22, 22, 22), (2, 2, 2)), (40, (17, 17, 17), (2, 2, 2))):
        d_mf = torch.from_numpy(np.maximum(synth.uniform_pm1(1003, 0, (maps,) + n), 0)).to("cuda:0")
        o = tuple(a - b + 1 for a, b in zip(n, win))
        d_mfg = torch.from_numpy(synth.uniform_pm1(1003, 2, (maps,) + o)).to("cuda:0")
        _, idx = znn.maxfilter3d_fwd(d_mf, win)
        work = rl.maxfilter_work(maps, n, win)
        for what, fn in (("MF-fwd", lambda: znn.maxfilter3d_fwd(d_mf, win)),
                         ("MF-bwd", lambda: znn.maxfilter3d_bwd(d_mfg, idx, n, win))):
            rec, treps = timer.trace(fn, 5)
            steps = rl.steps_of_pass(rec, treps, None, None, None, what, work)
            rows.append({"config": "C3", "layer": "max-filter %s on %dx%s" % ("x".join(map(str, win)), maps, "x".join(map(str, n))),
                         "mode": "-", "pass": what, "ms": steps[0]["ms"],
                         "frac_note": "not meaningful: microsecond kernel, bound by launch latency",
                         **{k: steps[0][k] for k in ("bound", "achieved", "peak", "unit", "frac") if k in steps[0]}})
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true", help="skip the per-configuration table")
    ap.add_argument("--probe", choices=["c5-fft", "c5-fft-full", "c2", "c4", "c2-direct"], default=None,
                    help="for rocprofv3 counter runs: run the named passes a few times, then a plain 1 GiB "
                         "device copy whose known size calibrates the byte counters, and exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1510_06706_amd import binding as znn
    from paper_1510_06706_amd import roofline as rl
    from paper_1510_06706_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    if args.probe:
        return probe(args.probe)

    timer = Timer(args.warmup, args.steps)
    cfg = synth.CONFIG5
    t0 = time.perf_counter()
    # ---- config 5: per-pass table in every variant (also generates its tensors, once)
    c5_rows, (inp, w, gout), (d_in, d_w, d_g), (out, gin, gw) = layer_rows(
        timer, cfg, "C5", [] if args.headline_only else
        [("fft", "folded", True, True), ("fft", "full", True, True), ("direct", None, False, False)])
    log("config 5 tensors and table: %.1f s" % (time.perf_counter() - t0))

    # ---- the per-layer choice between the methods (Section 4), measured on this shape
    chosen, tune_ms = znn.autotune(cfg.fan_in, cfg.fan_out, cfg.image, cfg.kernel)
    method = "fft" if chosen == znn.ZNN_FFT else "direct"
    log("autotune on config 5: %s (direct %.2f ms, fft %.2f ms per round without resident spectra)"
        % (method, sum(tune_ms[0]), sum(tune_ms[1])))
    torch.cuda.empty_cache()
    plan = znn.Plan(cfg.fan_in, cfg.fan_out, cfg.image, cfg.kernel, "auto")
    assert plan.mode == chosen
    if method == "fft":
        plan.enable_memo(dev)

    def step():
        if method == "fft":       # the memoized schedule of Section 4: every spectrum is computed once per round
            plan.prepare_kernels(d_w)
            plan.fwd(d_in, None, out)
            plan.bwd(d_g, None, gin)
            plan.wgrad_memo(gw)
        else:
            plan.fwd(d_in, d_w, out)
            plan.bwd(d_g, d_w, gin)
            plan.wgrad(d_in, d_g, gw)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # ---- kernels of the headline step, from HIP events the library records around every launch on the
    # stream it launches on; roofline of the one that takes the largest share of the step
    rec, treps = timer.trace(step, 3)
    layout = plan.spectra_layout if method == "fft" else None
    N = plan.fft_extents
    agg = {}
    for name, ms in rec:
        n_, t_ = agg.get(name, (0, 0.0))
        agg[name] = (n_ + 1, t_ + ms)
    kernels = [{"kernel": k, "launches_per_step": n_ / treps, "ms_per_launch": t_ / n_, "ms_per_step": t_ / treps}
               for k, (n_, t_) in agg.items()]
    top = max(kernels, key=lambda r: r["ms_per_step"])
    what = {"spectral mac forward": "fwd", "spectral mac backward": "bwd"}.get(top["kernel"].split(" (")[0], "wgrad_memo")
    if top["kernel"].startswith("direct forward"):
        what = "fwd"
    elif top["kernel"].startswith("direct backward"):
        what = "bwd"
    key = rl.step_of(top["kernel"], what)
    if key == "F-mac" and "MFMA" in top["kernel"]:
        key = "F-mac/mfma"
    bound, work = rl.work_of(cfg, N, layout or "folded", what)[key]
    roof = {"kernel": top["kernel"], "ms": top["ms_per_launch"], "launches_per_step": top["launches_per_step"]}
    roof.update(rl.price(bound, work, top["ms_per_launch"]))
    roof["algorithmic_work_per_launch"] = work
    traffic = rl.measured_traffic(TRAFFIC_PROFILE)
    roof["traffic"] = traffic.get(top["kernel"])
    roof["traffic_source"] = (TRAFFIC_PROFILE + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run, "
                              "scaled by a plain copy; not measured by this run)") if roof["traffic"] else None

    per_mode = {}
    for r in c5_rows:
        key = r["mode"] + ("" if r["mode"] == "direct" else ", " + r["kernel_spectra"])
        per_mode.setdefault(key, {"ms": {}})["ms"][r["pass"]] = round(r["ms"], 4)
    for key, v in per_mode.items():
        t = v["ms"]
        tot = sum(x for k, x in t.items() if k != ("wgrad" if "wgrad_memo" in t else ""))
        v["layer_ms"] = round(tot, 4)
        v["voxels_per_s"] = cfg.out_voxels / (tot * 1e-3)
        v["effective_tflops"] = 3 * 2.0 * cfg.macs / (tot * 1e-3) / 1e12

    result = {
        "metric": "conv-layer fwd+bwd+wgrad output voxels/s",
        "value": cfg.out_voxels / (ms_per_step * 1e-3),
        "unit": "output voxels/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "config 5: wide 3D layer f=120 -> f'=120, n=96^3, k=7^3, n'=90^3, one training round "
                               "(kernel transforms + forward + backward + kernel gradient) by the method the autotuner "
                               "picks: " + (("FFT, kernel spectra resident in HBM as " + layout + " spectra, node spectra memoized")
                                            if method == "fft" else "direct"),
                   "global_batch": 1, "method": method, "kernel_spectra": layout,
                   "autotune_ms": {"direct": [round(v, 3) for v in tune_ms[0]], "fft": [round(v, 3) for v in tune_ms[1]]}},
        "effective_tflops": 3 * 2.0 * cfg.macs / (ms_per_step * 1e-3) / 1e12,
        "per_mode": per_mode,
        "roofline": roof,
        "kernels": kernels,
    }
    plan.close()
    if not args.no_cpu_baseline:
        t0 = time.perf_counter()
        result["cpu_baseline"] = cpu_baseline(cfg, inp, w, gout)
        log("cpu baseline: %.1f s" % (time.perf_counter() - t0))
    del d_in, d_w, d_g, out, gin, gw, inp, w, gout
    torch.cuda.empty_cache()

    if not args.headline_only:
        rows = []
        variants = [("direct", None, False, False), ("fft", None, True, True)]
        rows += layer_rows(timer, synth.CONFIG1, "C1", variants, meaningful=False)[0]
        rows += layer_rows(timer, synth.CONFIG2, "C2", variants + [("fft", "full", True, True)])[0]
        rows += config3_rows(timer)
        rows += layer_rows(timer, synth.CONFIG4, "C4", variants + [("fft", "full", True, True)])[0]
        rows += c5_rows
        result["configs"] = rows
        result["configs_note"] = ("per pass: ms = mean of timed_reps launches after warm-up (HIP events on the launch stream; "
                                  "slow passes are capped at about 1.5 s of timed work), effective_tflops = 2 f f' n'^3 k^3 / t "
                                  "in either method; bound/achieved/frac are those of dominant_step, `steps` prices every step of "
                                  "the pass from the library's per-launch events; fft rows: kernel_spectra = the transforms of all "
                                  "kernels (once per round), wgrad_memo = kernel gradient from the node spectra forward and "
                                  "backward left behind, wgrad = the same with its own node transforms")
    print(json.dumps(result))


def probe(which):
    """Workloads for `rocprofv3 --pmc ... -- python3 bench.py --probe <which>` (counter runs)."""
    import torch
    from paper_1510_06706_amd import binding as znn
    from paper_1510_06706_amd import synth
    dev = torch.device("cuda:0")
    cfg = {"c5-fft": synth.CONFIG5, "c5-fft-full": synth.CONFIG5, "c2": synth.CONFIG2, "c2-direct": synth.CONFIG2,
           "c4": synth.CONFIG4}[which]
    inp, w, gout = synth.layer_tensors(cfg)
    d_in, d_w, d_g = (torch.from_numpy(a).to(dev) for a in (inp, w, gout))
    modes = ["fft"] if which.startswith("c5") else ["direct"] if which == "c2-direct" else ["direct", "fft"]
    for mode in modes:
        p = znn.Plan(cfg.fan_in, cfg.fan_out, cfg.image, cfg.kernel, mode)
        if mode == "fft":
            if which == "c5-fft-full":
                p.set_spectra_layout("full")
            p.enable_memo(dev)
        for _ in range(2):
            if mode == "fft":
                p.prepare_kernels(d_w)
                p.fwd(d_in, None); p.bwd(d_g, None); p.wgrad_memo()
            else:
                p.fwd(d_in, d_w); p.bwd(d_g, d_w); p.wgrad(d_in, d_g)
        torch.cuda.synchronize()
        p.close()
    a = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
    b = torch.empty_like(a)
    b.copy_(a)          # plain copy kernel: reads 1 GiB, writes 1 GiB
    torch.cuda.synchronize()
    print(json.dumps({"probe": which, "rounds": 2, "copy_bytes_each_way": a.numel() * 4}))


if __name__ == "__main__":
    main()
