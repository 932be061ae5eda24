"""Host-side checks of the benchmark's roofline bookkeeping (no GPU): the work model reproduces the
closed forms of Table 2 and of the kernels' own operation counts, launches are grouped into the right
steps, and the committed traffic profile parses."""
import os

from paper_1510_06706_amd import roofline as rl
from paper_1510_06706_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_work_model_closed_forms():
    c2, c5 = synth.CONFIG2, synth.CONFIG5
    w = rl.work_of(c2, (64, 64, 64), "full", "fwd")
    assert w["D-fwd"] == ("mfma", 2.0 * 40 * 40 * 60 ** 3 * 125) == ("mfma", 86.4e9)
    sv = 64 * 64 * 33
    assert w["F-mac"] == ("hbm", 8.0 * sv * (1600 + 80))                  # 8 bytes per kernel-spectrum element, once
    assert w["F-img"] == ("hbm", 40 * (4.0 * 64 ** 3 + 8.0 * sv))
    assert w["F-inv"] == ("hbm", 40 * (8.0 * sv + 4.0 * 60 ** 3))
    w5 = rl.work_of(c5, (96, 96, 96), "full", "bwd")
    assert w5["F-ker"][1] == 4.0 * 14400 * 343 + 52022476800.0           # 52.02 GB of full spectra
    f5 = rl.work_of(c5, (96, 96, 96), "folded", "wgrad_memo")
    sv5 = 96 * 96 * 49
    assert f5["F-ker"][1] == 4.0 * 14400 * 343 + 8.0 * 14400 * 7 * 96 * 49
    assert f5["F-mac"] == ("alu", 14400 * sv5 / 4.0 * (6 * 6 + 2 * 3 + 48))
    assert f5["F-mac/mfma"] == ("alu", 14400 * sv5 / 4.0 * 48 + 14400 * 294 * 3 * 4 * 2048.0)
    assert f5["F-wgrad z"] == ("alu", 14400 * sv5 / 4.0 * 90)
    assert f5["F-wgrad y"] == ("hbm", 8.0 * 14400 * 7 * 96 * 49 + 8.0 * 14400 * 49 * 49)
    # 2D: the first contracted axis is y, there is no second pruned axis
    w4 = rl.work_of(synth.CONFIG4, (1, 256, 256), "folded", "wgrad")
    assert "F-wgrad y" not in w4 and w4["F-wgrad z"][1] == 6400 * 256 * 129 / 4.0 * (42 + 80)


def test_mfma_step_counts_of_the_class_sums():
    # classes a mod 4 with t taps take ceil(2 t / 4) k-steps
    assert [rl.mfma_steps(k) for k in (1, 2, 3, 4, 5, 7, 8, 9, 11, 16)] == [1, 2, 3, 4, 4, 4, 4, 5, 7, 8]


def test_launches_are_grouped_into_steps_and_priced():
    rec = [("fft r2c x (registers)", 0.2), ("fft axis forward (registers)", 0.2), ("fft axis forward (registers)", 0.2),
           ("spectral mac forward (taps folded in, MFMA)", 2.6), ("fft axis inverse (registers)", 0.2),
           ("fft axis inverse (registers)", 0.2), ("fft c2r x (registers)", 0.2)] * 2
    rows = rl.steps_of_pass(rec, 2, synth.CONFIG5, (96, 96, 96), "folded", "fwd")
    assert [r["step"] for r in rows] == ["F-img", "F-mac", "F-inv"]
    assert [r["launches"] for r in rows] == [3, 1, 3]
    mac = rows[1]
    assert mac["bound"] == "alu" and abs(mac["ms"] - 2.6) < 1e-12
    assert abs(mac["achieved"] - 182078668800.0 / 2.6e-3 / 1e12) < 1e-9
    assert abs(mac["frac"] * 157.3 - mac["achieved"]) < 1e-9 and abs(mac["frac_of_unpacked_peak"] * 78.6 - mac["achieved"]) < 1e-9
    assert rl.dominant(rows)["step"] == "F-mac"
    img = rows[0]
    assert img["bound"] == "hbm" and abs(img["achieved"] - 120 * (4.0 * 96 ** 3 + 8.0 * 96 * 96 * 49) / 0.6e-3 / 1e9) < 1e-6
    # the same kernel name is the x axis of the kernel gradient in a gradient pass
    assert rl.step_of("fft c2r x (registers)", "wgrad_memo") == "F-wgrad x"
    assert rl.step_of("direct kernel gradient (MFMA)", "wgrad") == "D-wgrad"
    assert rl.step_of("fft r2c x", "kernel_spectra") == "F-ker"


def test_committed_traffic_profile_parses():
    t = rl.measured_traffic("profiles/config5_hbm_traffic_pmc.txt")
    assert os.path.exists(os.path.join(ROOT, "profiles", "config5_hbm_traffic_pmc.txt"))
    assert t and all(v > 0 for v in t.values())
    assert any(k.startswith("spectral mac forward") for k in t)
    assert rl.measured_traffic("profiles/no_such_file.txt") == {}
