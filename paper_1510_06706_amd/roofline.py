"""Roofline bookkeeping for the benchmark: the algorithmic work of every step of the hot path
and the published MI355X peaks it is priced against.  No compute happens here.

Steps (rows of the hot path) and what bounds them:

  D-fwd / D-bwd / D-wgrad   fp32 matrix cores; 2 FLOP per multiply-add, f f' n'^3 k^3 of them per pass
                            (Table 2, "Direct", which counts a multiply-add once).
  F-img / F-inv             HBM; per node volume one read of the image (4 n^3 bytes; 4 n'^3 for an output
                            gradient) and one write of its spectrum (8 N_w bytes), resp. the reverse.
  F-ker                     HBM; the kernel spectra are written once in the plan's layout.
  F-mac, full spectra       HBM; every kernel-spectrum element is streamed once (8 bytes) and used in one
                            complex multiply-add (8 FLOP); node spectra read and written once.
  F-mac, half spectra       fp32 vector ALU.  FLOPs are the ones the kernel executes: a thread handles
                            four frequencies a quarter period apart at a time, per edge
                              (taps-1) complex multiplications by twiddles   6 FLOP each
                              max(taps-4, 0) complex additions (folding taps by index mod 4)   2 each
                              radix-4 butterfly of 8 complex additions       16
                              4 complex multiply-adds with the node spectrum 32
                            -> flops4 = 6 (taps-1) + 2 max(taps-4, 0) + 48 per edge and 4 frequencies.
  F-mac, half spectra,      the same with the class sums V_c[z0] = sum_{a = c mod 4} Wh[a] exp(-2 pi i a z0 / N)
  rebuild on matrix cores   taken by v_mfma_f32_16x16x4_f32 (per edge, 16 in-plane frequencies and 8 z0: one MFMA
                            per class and per two taps of the class, 2048 FLOP each, padding rows included) and
                            only the radix-4 butterfly (16) and the four complex multiply-adds (32) left on the
                            vector ALUs: 48 FLOP per edge and 4 frequencies.  On this chip an MFMA and vector
                            instructions of the same SIMD take turns rather than overlap (measured: busy cycles
                            of the two add up to the elapsed time), so the row is priced on the sum of both
                            kinds of executed FLOPs against the one 157.3 TFLOP/s that either unit peaks at.
  F-wgrad z                 fp32 vector ALU (pruned DFT of the spectral products).  Per pair of nodes and
                            four z a quarter period apart: 4 products g conj(x) (6 FLOP), a radix-4
                            butterfly (16), one complex addition (2) and taps-1 complex multiply-adds (8):
                              flops4 = 42 + 8 (taps-1).
                            Layers that cannot group by four run taps complex multiply-adds per z.
  F-wgrad y                 HBM; reads the z-contracted pair volumes once, writes k_y rows of each.
  F-wgrad x                 HBM; c2r of k_z k_y rows per pair.
  MF-fwd / MF-bwd           HBM; 4 bytes read + 8 written per output voxel, resp. 8 read + 4 written per
                            input voxel.

Peaks: fp32 MFMA 157.3 TFLOP/s; HBM 8 TB/s; fp32 vector 157.3 TFLOP/s = 256 CUs x 4 SIMDs x 16 lanes x
2 (packed) x 2 FLOP x 2.4 GHz.  This build issues no packed fp32 instructions (compiler flag required on
this pool), which caps the vector ALUs at 78.6 TFLOP/s; rows bound by them carry both fractions.
"""
from __future__ import annotations

import os
from collections import OrderedDict

PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_FP32_VECTOR_TFLOPS = 157.3
PEAK_FP32_VECTOR_UNPACKED_TFLOPS = 78.6
PEAK_HBM_GBS = 8000.0

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def spectrum_elems(N) -> int:
    return N[0] * N[1] * (N[2] // 2 + 1)


def flops4_mac_folded(taps: int) -> float:
    return 6.0 * (taps - 1) + 2.0 * max(taps - 4, 0) + 48.0


def mfma_steps(taps: int) -> int:
    """MFMA k-steps per (edge, 16 p, 8 z0) of the class sums: ceil(2 * taps_of_class / 4) over the four classes."""
    return sum((2 * ((taps - c + 3) // 4) + 3) // 4 for c in range(4) if c < taps)


def flops4_wgrad_dft(taps: int) -> float:
    return 42.0 + 8.0 * (taps - 1)


# kernel role (name the library records per launch) -> step of the hot path, per pass
def step_of(name: str, what: str) -> str:
    if name.startswith("direct forward"):
        return "D-fwd"
    if name.startswith("direct backward"):
        return "D-bwd"
    if name.startswith("direct kernel gradient"):
        return "D-wgrad"
    if name in ("weight packing", "sum over input-map shares", "kernel gradient reduction"):
        return "direct: packing and fixed-order sums"
    if name.startswith("spectral mac"):
        return "F-mac"
    if name == "pruned DFT of spectral products" or name.endswith("of product"):
        return "F-wgrad z"
    if name.startswith("pruned DFT, second axis"):
        return "F-wgrad y"
    if what == "kernel_spectra":
        return "F-ker"
    if name.startswith("fft c2r"):
        return "F-wgrad x" if what == "wgrad_memo" or what == "wgrad" else "F-inv"
    if name.startswith("fft axis inverse"):
        return "F-wgrad y" if what in ("wgrad", "wgrad_memo") else "F-inv"
    if name.startswith("fft r2c x") or name == "pruned z DFT of kernels" or name.startswith("fft axis forward"):
        return "F-img"
    if name == "max-filter forward":
        return "MF-fwd"
    if name == "max-filter backward":
        return "MF-bwd"
    return name


def work_of(cfg, N, layout: str, what: str):
    """{step: (bound, algorithmic work per pass)}: FLOP for "mfma"/"alu", bytes for "hbm".

    cfg: layer shape; N: FFT extents; layout: "full" | "folded" (kernel spectra);
    what: "fwd" | "bwd" | "wgrad" | "wgrad_memo" | "kernel_spectra".
    """
    f, fo = cfg.fan_in, cfg.fan_out
    n = 1
    for v in cfg.image:
        n *= v
    no = 1
    for v in cfg.out:
        no *= v
    kz, ky, kx = cfg.kernel
    sv = spectrum_elems(N)
    pairs = f * fo
    Nxh = N[2] // 2 + 1
    threeD = N[0] > 1
    taps = kz if threeD else ky
    Nfold = N[0] if threeD else N[1]
    sparse_fold = (cfg.sparsity[0] if threeD else cfg.sparsity[1]) != 1
    flops = 2.0 * cfg.macs
    w = OrderedDict()
    w["D-fwd"] = ("mfma", flops)
    w["D-bwd"] = ("mfma", flops)
    w["D-wgrad"] = ("mfma", flops)
    if layout == "folded":
        kspec = 8.0 * pairs * taps * (sv // Nfold)
        w["F-mac"] = ("alu", pairs * sv / 4.0 * flops4_mac_folded(taps))
        ptiles = -(-(sv // Nfold) // 16)
        w["F-mac/mfma"] = ("alu", pairs * sv / 4.0 * 48.0 + pairs * ptiles * (Nfold // 32) * mfma_steps(taps) * 2048.0)
    else:
        kspec = 8.0 * pairs * sv
        w["F-mac"] = ("hbm", 8.0 * sv * (pairs + f + fo))
    w["F-ker"] = ("hbm", 4.0 * pairs * kz * ky * kx + kspec)
    if what == "fwd":
        w["F-img"] = ("hbm", f * (4.0 * n + 8.0 * sv))
        w["F-inv"] = ("hbm", fo * (8.0 * sv + 4.0 * no))
    elif what == "bwd":
        w["F-img"] = ("hbm", fo * (4.0 * no + 8.0 * sv))
        w["F-inv"] = ("hbm", f * (8.0 * sv + 4.0 * n))
    else:
        w["F-img"] = ("hbm", f * (4.0 * n + 8.0 * sv) + fo * (4.0 * no + 8.0 * sv))
    grouped = Nfold % 4 == 0 and not sparse_fold
    w["F-wgrad z"] = ("alu", pairs * sv / 4.0 * flops4_wgrad_dft(taps) if grouped else pairs * sv * 8.0 * taps)
    if threeD:
        t1 = 8.0 * pairs * kz * N[1] * Nxh
        t2 = 8.0 * pairs * kz * ky * Nxh
        w["F-wgrad y"] = ("hbm", t1 + t2)
    else:
        t2 = 8.0 * pairs * ky * Nxh
    w["F-wgrad x"] = ("hbm", t2 + 4.0 * pairs * kz * ky * kx)
    return w


def maxfilter_work(maps, n, win):
    vin, vout = maps, maps
    for a, b in zip(n, win):
        vin *= a
        vout *= a - b + 1
    return {"MF-fwd": ("hbm", 4.0 * vin + 8.0 * vout), "MF-bwd": ("hbm", 8.0 * vout + 4.0 * vin)}


def price(bound: str, work: float, ms: float):
    """Achieved rate and fraction(s) of the published peak for `work` done in `ms`."""
    if ms <= 0.0:
        return {}
    if bound == "hbm":
        a = work / (ms * 1e-3) / 1e9
        return {"bound": "hbm", "achieved": a, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": a / PEAK_HBM_GBS}
    a = work / (ms * 1e-3) / 1e12
    if bound == "mfma":
        return {"bound": "mfma", "achieved": a, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": a / PEAK_FP32_MFMA_TFLOPS}
    return {"bound": "alu", "achieved": a, "peak": PEAK_FP32_VECTOR_TFLOPS, "unit": "TFLOP/s",
            "frac": a / PEAK_FP32_VECTOR_TFLOPS, "frac_of_unpacked_peak": a / PEAK_FP32_VECTOR_UNPACKED_TFLOPS,
            "work": "FLOPs the kernel executes"}


def steps_of_pass(records, reps, cfg, N, layout, what, extra_work=None):
    """records: [(kernel role, ms)] of `reps` traced runs of one pass -> [{step, kernels, launches, ms, ...}]
    with every step priced against its roofline, in launch order of first appearance."""
    model = dict(work_of(cfg, N, layout, what)) if cfg is not None else {}
    if extra_work:
        model.update(extra_work)
    agg = OrderedDict()
    for name, ms in records:
        st = step_of(name, what)
        e = agg.setdefault(st, {"step": st, "kernels": [], "launches": 0, "ms": 0.0})
        if name not in e["kernels"]:
            e["kernels"].append(name)
        e["launches"] += 1
        e["ms"] += ms
    rows = []
    for st, e in agg.items():
        e["launches"] = e["launches"] / reps
        e["ms"] = e["ms"] / reps
        key = st + "/mfma" if st == "F-mac" and any("MFMA" in k for k in e["kernels"]) else st
        if key in model:
            e.update(price(model[key][0], model[key][1], e["ms"]))
            if key.endswith("/mfma"):
                e["work"] = "FLOPs the kernel executes: vector ALU (butterfly, product) + matrix cores (class sums)"
        rows.append(e)
    return rows


def dominant(rows):
    """The priced step that takes the most time."""
    priced = [r for r in rows if "frac" in r]
    return max(priced, key=lambda r: r["ms"]) if priced else None


def measured_traffic(path):
    """HBM bytes per launch (read + written) from a committed rocprofv3 counter summary: lines of the form
    `traffic: <kernel role> | <read bytes> | <written bytes>`.  {} when the file is missing."""
    out = {}
    try:
        with open(os.path.join(ROOT, path)) as fh:
            for line in fh:
                if line.startswith("traffic:"):
                    name, rd, wr = (t.strip() for t in line[len("traffic:"):].split("|"))
                    out[name] = float(rd) + float(wr)
    except OSError:
        pass
    return out
