"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol include/znn.h declares, and validates its arguments before launching anything."""
import ctypes
import os
import re

import pytest

from paper_1510_06706_amd import binding as znn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "znn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(znn_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = znn.lib()
    names = declared_symbols()
    assert len(names) >= 20
    for n in names:
        assert hasattr(L, n), n
    assert sorted(znn.EXPORTS) == names


def plan_rc(**kw):
    d = dict(fan_in=2, fan_out=3, image=(4, 5, 6), kernel=(2, 2, 3), mode="direct", sparsity=(1, 1, 1))
    d.update(kw)
    desc = znn.make_desc(d["fan_in"], d["fan_out"], d["image"], d["kernel"], d["mode"], d["sparsity"])
    h = ctypes.c_void_p(0)
    rc = znn.lib().znn_plan_create(ctypes.byref(desc), ctypes.byref(h))
    if rc == 0:
        znn.lib().znn_plan_destroy(h)
    return rc


def test_descriptor_validation():
    assert plan_rc() == znn.ZNN_OK
    assert plan_rc(fan_in=0) == znn.ZNN_EINVAL
    assert plan_rc(fan_out=-1) == znn.ZNN_EINVAL
    assert plan_rc(kernel=(5, 2, 3)) == znn.ZNN_EINVAL
    assert "exceeds" in znn.last_error()
    assert plan_rc(image=(0, 5, 6)) == znn.ZNN_EINVAL
    assert plan_rc(kernel=(1, 0, 1)) == znn.ZNN_EINVAL
    assert plan_rc(sparsity=(2, 2, 2)) == znn.ZNN_OK          # spans 3, 3, 5 fit 4, 5, 6
    assert plan_rc(sparsity=(4, 1, 1)) == znn.ZNN_EINVAL      # span 5 exceeds 4
    assert plan_rc(sparsity=(0, 1, 1)) == znn.ZNN_EINVAL
    assert plan_rc(mode=7) == znn.ZNN_EINVAL
    assert plan_rc(mode="fft", image=(1, 4, 2000), kernel=(1, 1, 1)) == znn.ZNN_EUNSUPPORTED
    assert znn.lib().znn_plan_create(None, ctypes.byref(ctypes.c_void_p(0))) == znn.ZNN_EINVAL


@pytest.mark.parametrize("n,N", [((16, 16, 16), (16, 16, 16)), ((26, 22, 17), (27, 24, 18)),
                                 ((1, 256, 246), (1, 256, 250)), ((96, 90, 7), (96, 90, 8))])
def test_fft_extents_are_the_next_5_smooth_numbers(n, N):
    p = znn.Plan(1, 1, n, (1, 1, 1), "fft")
    assert p.fft_extents == N
    assert p.mode == znn.ZNN_FFT
    p.close()


def test_workspace_and_spectra_sizes():
    p = znn.Plan(40, 40, (64, 64, 64), (5, 5, 5), "fft")
    spec = 64 * 64 * 33 * 8
    # kernels are kept transformed along y and x only: 5 planes of taps instead of 64
    kspec = 40 * 40 * 5 * 64 * 33 * 8
    assert p.spectra_bytes() == kspec
    assert p.workspace_bytes(znn.ZNN_PASS_FWD) == 80 * spec + kspec
    assert p.workspace_bytes(znn.ZNN_PASS_BWD) == 80 * spec + kspec
    assert p.workspace_bytes(znn.ZNN_PASS_WGRAD) >= 80 * spec
    p.close()
    # a small layer, an extent not divisible by 4 and taps more than one voxel apart along z
    # keep full spectra
    for n, k, s, N in (((12, 12, 12), (3, 3, 3), (1, 1, 1), (12, 12, 12)),
                       ((26, 64, 64), (5, 5, 5), (1, 1, 1), (27, 64, 64)),
                       ((64, 64, 64), (5, 5, 5), (2, 1, 1), (64, 64, 64))):
        p = znn.Plan(40, 40, n, k, "fft", s)
        assert p.spectra_bytes() == 40 * 40 * N[0] * N[1] * (N[2] // 2 + 1) * 8, (n, k, s)
        p.close()
    p = znn.Plan(80, 80, (1, 256, 256), (1, 11, 11), "fft")       # 2D: the y axis is the folded one
    assert p.spectra_bytes() == 80 * 80 * 11 * 129 * 8
    b = ctypes.c_size_t(0)
    assert znn.lib().znn_plan_workspace_bytes(p._h, 5, ctypes.byref(b)) == znn.ZNN_EINVAL
    p.close()
    d = znn.Plan(40, 40, (64, 64, 64), (5, 5, 5), "direct")
    assert d.mode == znn.ZNN_DIRECT
    d.close()


def test_compute_entry_points_reject_null_and_short_workspace_without_launching():
    L = znn.lib()
    p = znn.Plan(2, 2, (8, 8, 8), (3, 3, 3), "fft")
    null = ctypes.c_void_p(0)
    fake = ctypes.c_void_p(0x1000)     # never dereferenced: validation fails first
    assert L.znn_conv3d_fwd(p._h, null, fake, fake, fake, 1 << 30, null) == znn.ZNN_EINVAL
    assert L.znn_conv3d_fwd(p._h, fake, fake, fake, null, 0, null) == znn.ZNN_EWORKSPACE
    assert L.znn_conv3d_bwd(p._h, fake, fake, fake, fake, 16, null) == znn.ZNN_EWORKSPACE
    assert L.znn_conv3d_wgrad(p._h, fake, fake, fake, ctypes.c_void_p(0x1001), 1 << 30, null) == znn.ZNN_EWORKSPACE
    assert "aligned" in znn.last_error()
    assert L.znn_conv_prepare_kernels(p._h, fake, null, 0, null, 0, null) == znn.ZNN_EWORKSPACE
    p.close()
    d = znn.Plan(2, 2, (8, 8, 8), (3, 3, 3), "direct")
    assert L.znn_conv_prepare_kernels(d._h, fake, fake, 1 << 30, null, 0, null) == znn.ZNN_EINVAL
    d.close()


def test_filter_and_pointwise_validation():
    L = znn.lib()
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    v = znn.Vec3
    assert L.znn_maxfilter3d_fwd(1, v(4, 4, 4), v(5, 1, 1), fake, fake, fake, null) == znn.ZNN_EINVAL
    assert L.znn_maxfilter3d_fwd(0, v(4, 4, 4), v(2, 2, 2), fake, fake, fake, null) == znn.ZNN_EINVAL
    assert L.znn_maxfilter3d_fwd(1, v(4, 4, 4), v(2, 2, 2), null, fake, fake, null) == znn.ZNN_EINVAL
    assert L.znn_maxfilter3d_bwd(1, v(4, 4, 4), v(2, 0, 2), fake, fake, fake, null) == znn.ZNN_EINVAL
    assert L.znn_maxfilter3d_fwd(1, v(2048, 2048, 1024), v(2, 2, 2), fake, fake, fake, null) == znn.ZNN_EUNSUPPORTED
    one = v(1, 1, 1)
    assert L.znn_maxfilter3d_sparse_fwd(1, v(4, 4, 4), v(2, 2, 2), v(4, 1, 1), fake, fake, fake, null) == znn.ZNN_EINVAL
    assert L.znn_maxfilter3d_sparse_fwd(1, v(5, 4, 4), v(2, 2, 2), v(0, 1, 1), fake, fake, fake, null) == znn.ZNN_EINVAL
    assert L.znn_maxfilter3d_sparse_bwd(1, v(5, 4, 4), v(2, 2, 2), v(4, 1, 1), null, fake, fake, null) == znn.ZNN_EINVAL
    assert L.znn_maxfilter3d_sparse_bwd(1, v(4, 4, 4), v(2, 2, 2), one, fake, fake, null, null) == znn.ZNN_EINVAL
    assert L.znn_maxpool3d_fwd(1, v(5, 4, 4), v(2, 2, 2), fake, fake, fake, null) == znn.ZNN_EINVAL
    assert "divisible" in znn.last_error()
    assert L.znn_maxpool3d_fwd(1, v(4, 4, 4), v(2, 2, 2), fake, null, fake, null) == znn.ZNN_EINVAL
    assert L.znn_maxpool3d_bwd(1, v(4, 4, 4), v(2, 0, 2), fake, fake, fake, null) == znn.ZNN_EINVAL
    assert L.znn_transfer_fn_fwd(3, 1, 10, fake, fake, fake, null) == znn.ZNN_EINVAL
    assert L.znn_transfer_fn_bwd(-1, 1, 10, fake, fake, fake, null) == znn.ZNN_EINVAL
    assert L.znn_transfer_fn_fwd(1, 1, 10, null, fake, fake, null) == znn.ZNN_EINVAL
    assert L.znn_cross_entropy_loss_grad(0, fake, fake, fake, null) == znn.ZNN_EINVAL
    assert L.znn_cross_entropy_loss_grad(5, fake, null, fake, null) == znn.ZNN_EINVAL
    assert L.znn_transfer_fwd(0, 10, fake, fake, fake, null) == znn.ZNN_EINVAL
    assert L.znn_bias_grad(2, 10, null, fake, null) == znn.ZNN_EINVAL
    assert L.znn_sgd_update(0, 0.1, fake, fake, null) == znn.ZNN_EINVAL


def test_auto_mode_resolves_to_a_concrete_method():
    p = znn.Plan(120, 120, (96, 96, 96), (7, 7, 7), "auto")
    assert p.mode in (znn.ZNN_DIRECT, znn.ZNN_FFT)
    p.close()


def test_memo_entry_points_validate_their_state():
    L = znn.lib()
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    d = znn.Plan(2, 2, (8, 8, 8), (3, 3, 3), "direct")
    assert L.znn_conv_set_memo(d._h, fake, 1 << 30) == znn.ZNN_EINVAL
    d.close()
    p = znn.Plan(2, 3, (8, 8, 8), (3, 3, 3), "fft")
    assert p.memo_bytes() == 5 * 8 * 8 * 5 * 8
    assert L.znn_conv3d_wgrad_memo(p._h, fake, fake, 1 << 30, null) == znn.ZNN_EINVAL     # nothing attached
    assert L.znn_conv_set_memo(p._h, fake, 16) == znn.ZNN_EWORKSPACE
    assert L.znn_conv_set_memo(p._h, ctypes.c_void_p(0x1001), 1 << 30) == znn.ZNN_EWORKSPACE
    assert L.znn_conv_set_memo(p._h, fake, 1 << 30) == znn.ZNN_OK
    assert L.znn_conv3d_wgrad_memo(p._h, fake, fake, 1 << 30, null) == znn.ZNN_EINVAL     # passes have not run
    assert "forward and the backward" in znn.last_error()
    assert L.znn_conv_set_memo(p._h, null, 0) == znn.ZNN_OK
    p.close()


def test_round_autotuner_validates_before_launching():
    L = znn.lib()
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    d = znn.make_desc(4, 4, (12, 12, 12), (3, 3, 3), "auto")
    rep = znn.RoundReport()
    need, single = ctypes.c_size_t(0), ctypes.c_size_t(0)
    assert L.znn_autotune_round_workspace_bytes(ctypes.byref(d), ctypes.byref(need)) == znn.ZNN_OK
    assert L.znn_autotune_workspace_bytes(ctypes.byref(d), ctypes.byref(single)) == znn.ZNN_OK
    assert need.value >= single.value > 0
    assert L.znn_autotune_round_workspace_bytes(ctypes.byref(d), None) == znn.ZNN_EINVAL
    assert L.znn_autotune_round(ctypes.byref(d), 1 << 40, fake, need.value, null, None) == znn.ZNN_EINVAL
    assert L.znn_autotune_round(ctypes.byref(d), 0, fake, need.value, null, ctypes.byref(rep)) == znn.ZNN_EWORKSPACE
    assert "budget" in znn.last_error()
    assert rep.bytes[2] > rep.bytes[1] > rep.bytes[0] > 0 and rep.chosen == -1
    assert L.znn_autotune_round(ctypes.byref(d), 1 << 40, null, need.value, null, ctypes.byref(rep)) == znn.ZNN_EWORKSPACE
    assert L.znn_autotune_round(ctypes.byref(d), 1 << 40, fake, 16, null, ctypes.byref(rep)) == znn.ZNN_EWORKSPACE
    bad = znn.make_desc(4, 4, (2, 12, 12), (3, 3, 3), "auto")
    assert L.znn_autotune_round(ctypes.byref(bad), 1 << 40, fake, need.value, null, ctypes.byref(rep)) == znn.ZNN_EINVAL


def test_bench_refuses_more_than_one_gpu():
    """Every box of this build has one GPU: bench.py says so and exits instead of pretending to scale."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_spectra_layout_is_a_property_of_the_plan():
    """Full spectra (the paper's memoized kernel transforms, Section 4) or half spectra: chosen
    per plan through the ABI, reported back, and reflected in every size query."""
    p = znn.Plan(120, 120, (96, 96, 96), (7, 7, 7), "fft")
    spec = 96 * 96 * 49 * 8
    assert p.spectra_layout == "folded"
    assert p.spectra_bytes() == 120 * 120 * 7 * 96 * 49 * 8
    folded_ws = p.workspace_bytes(znn.ZNN_PASS_FWD)
    p.set_spectra_layout("full")
    assert p.spectra_layout == "full"
    assert p.spectra_bytes() == 120 * 120 * spec == 52022476800           # 52.02 GB
    assert p.workspace_bytes(znn.ZNN_PASS_FWD) == folded_ws + 120 * 120 * (96 - 7) * 96 * 49 * 8
    p.set_spectra_layout("folded")
    assert p.spectra_layout == "folded"
    p.set_spectra_layout("auto")
    assert p.spectra_layout == "folded"
    assert znn.lib().znn_plan_set_spectra_layout(p._h, 9) == znn.ZNN_EINVAL
    p.close()
    # a layer too small to fill the chip keeps full spectra by default but takes half spectra on request
    q = znn.Plan(1, 4, (16, 16, 16), (3, 3, 3), "fft")
    assert q.spectra_layout == "full"
    q.set_spectra_layout("folded")
    assert q.spectra_layout == "folded" and q.spectra_bytes() == 4 * 3 * 16 * 9 * 8
    q.close()
    # extents not divisible by 4 and sparse taps along the slowest axis cannot be folded
    r = znn.Plan(2, 2, (18, 16, 16), (3, 3, 3), "fft")
    assert znn.lib().znn_plan_set_spectra_layout(r._h, 2) == znn.ZNN_EUNSUPPORTED
    assert r.spectra_layout == "full"
    r.close()
    r = znn.Plan(2, 2, (16, 16, 16), (3, 3, 3), "fft", sparsity=(2, 1, 1))
    assert znn.lib().znn_plan_set_spectra_layout(r._h, 2) == znn.ZNN_EUNSUPPORTED
    r.close()
    d = znn.Plan(2, 2, (16, 16, 16), (3, 3, 3), "direct")
    assert znn.lib().znn_plan_set_spectra_layout(d._h, 1) == znn.ZNN_EINVAL
    d.close()
    assert znn.lib().znn_plan_set_spectra_layout(None, 1) == znn.ZNN_EINVAL
    assert znn.lib().znn_plan_spectra_layout(None, None) == znn.ZNN_EINVAL
