"""Roofline bookkeeping for the benchmark: algorithmic work of each pass and the
published MI355X peaks it is priced against.  No compute happens here."""
from __future__ import annotations

PEAK_FP32_MFMA_TFLOPS = 157.3   # dense fp32 matrix-core peak
PEAK_HBM_GBS = 8000.0           # HBM3E


def direct_pass_flops(cfg) -> float:
    """2 FLOP per multiply-add of the direct method, f * f' * n'^3 * k^3 of them (Table 2)."""
    return 2.0 * cfg.macs


def dominant(cfg, per, plans, *tensors):
    """Roofline entry of the kernel that takes the largest share of a step.

    Each direct pass is one kernel launch, so its event-timed duration is the kernel's.
    """
    name, ms = max(per["direct"].items(), key=lambda kv: kv[1])
    flops = direct_pass_flops(cfg)
    achieved = flops / (ms * 1e-3) / 1e12
    return {"kernel": "direct %s" % name, "bound": "mfma", "achieved": achieved,
            "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_FP32_MFMA_TFLOPS,
            "traffic": None, "ms": ms}
