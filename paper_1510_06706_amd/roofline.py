"""Roofline bookkeeping for the benchmark: algorithmic work of each kernel role and the
published MI355X peaks it is priced against.  No compute happens here."""
from __future__ import annotations

from collections import OrderedDict

PEAK_FP32_MFMA_TFLOPS = 157.3   # dense fp32 matrix-core peak
PEAK_FP32_VECTOR_TFLOPS = 157.3 # fp32 vector ALUs: 256 CUs x 4 SIMDs x 16 lanes x 2 (packed) x 2 FLOP x 2.4 GHz;
                                # this build issues no packed fp32 instructions, which halves what it can reach
PEAK_HBM_GBS = 8000.0           # HBM3E


# HBM bytes per launch (read, write) on the config-2 layer, from the rocprofv3 FETCH_SIZE /
# WRITE_SIZE runs summarised in profiles/config2_hbm_traffic_pmc.txt (counters scaled by a
# plain 1 GiB copy: x2.000 for FETCH_SIZE, x1.000 for WRITE_SIZE).  Static record of a
# separate profiler run, not measured by the benchmark itself.
MIB = 1024.0 * 1024.0
MEASURED_TRAFFIC_CONFIG2 = {
    "direct forward (MFMA)": (253.8 * MIB, 45.4 * MIB),
    "direct backward (MFMA)": (188.5 * MIB, 40.0 * MIB),
    "direct kernel gradient (MFMA)": (847.2 * MIB, 10.3 * MIB),
    "spectral mac forward (taps folded in)": (451.2 * MIB, 41.3 * MIB),
    "spectral mac backward (taps folded in)": (436.6 * MIB, 41.3 * MIB),
}


def spectrum_elems(N) -> int:
    return N[0] * N[1] * (N[2] // 2 + 1)


def work_model(cfg, N):
    """Algorithmic work per launch of the kernels that can dominate a step.

    direct passes: 2 FLOP per multiply-add, f f' n'^3 k^3 of them (Table 2, "Direct").
    spectral multiply-accumulate: every kernel-spectrum element is read once (8 B) and used
    in one complex multiply-add (8 FLOP); the node spectra are read / written once.
    """
    sv = spectrum_elems(N)
    mac_bytes = 8.0 * sv * (cfg.fan_in * cfg.fan_out + cfg.fan_in + cfg.fan_out)
    flops = 2.0 * cfg.macs
    # multiply-accumulate with the kernel transform's last axis folded in: per edge and
    # frequency, taps - 1 complex multiply-adds rebuild the kernel spectrum from its half
    # spectrum and one more forms the product, 8 FLOP each
    taps = cfg.kernel[0] if N[0] > 1 else cfg.kernel[1]
    folded_flops = 8.0 * taps * sv * cfg.fan_in * cfg.fan_out
    return {
        "direct forward (MFMA)": ("mfma", flops),
        "direct backward (MFMA)": ("mfma", flops),
        "direct kernel gradient (MFMA)": ("mfma", flops),
        "spectral mac forward": ("hbm", mac_bytes),
        "spectral mac backward": ("hbm", mac_bytes),
        "spectral mac forward (taps folded in)": ("alu", folded_flops),
        "spectral mac backward (taps folded in)": ("alu", folded_flops),
    }


def summarize(records, steps):
    """records: [(name, ms)] over `steps` traced steps -> {name: (launches per step, ms per launch)}."""
    agg = OrderedDict()
    for name, ms in records:
        n, t = agg.get(name, (0, 0.0))
        agg[name] = (n + 1, t + ms)
    return OrderedDict((k, (n / steps, t / n)) for k, (n, t) in agg.items())


def entry(name, ms, model, traffic=None):
    bound, work = model[name]
    if bound == "mfma":
        achieved, peak, unit = work / (ms * 1e-3) / 1e12, PEAK_FP32_MFMA_TFLOPS, "TFLOP/s"
    elif bound == "alu":
        achieved, peak, unit = work / (ms * 1e-3) / 1e12, PEAK_FP32_VECTOR_TFLOPS, "TFLOP/s"
    else:
        achieved, peak, unit = work / (ms * 1e-3) / 1e9, PEAK_HBM_GBS, "GB/s"
    return {"kernel": name, "bound": bound, "achieved": achieved, "peak": peak, "unit": unit,
            "frac": achieved / peak, "traffic": traffic, "ms": ms}


def report(cfg, N, records, steps):
    """(roofline of the dominant modelled kernel, per-kernel table)."""
    model = work_model(cfg, N)
    measured = MEASURED_TRAFFIC_CONFIG2 if cfg.name.startswith("c2_") else {}
    table = summarize(records, steps)
    kernels = []
    best = None
    for name, (per_step, ms) in table.items():
        row = {"kernel": name, "launches_per_step": per_step, "ms_per_launch": ms, "ms_per_step": per_step * ms}
        if name in model:
            t = measured.get(name)
            e = entry(name, ms, model, None if t is None else t[0] + t[1])
            row.update({"bound": e["bound"], "achieved": e["achieved"], "unit": e["unit"], "frac": e["frac"]})
            if best is None or per_step * ms > best[0]:
                best = (per_step * ms, e)
        kernels.append(row)
    return (best[1] if best else None), kernels
