"""Parity of the HIP library with the CPU oracle, element by element, through the C ABI.

Tolerances are the ones the task fixes: max|gpu - ref| / max|ref| <= 1e-4 for the
direct method and <= 1e-3 for the FFT method; max-filter values and indices are exact.
"""
import numpy as np
import pytest

import oracle
from paper_1510_06706_amd import binding as znn
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
    return float(np.max(np.abs(got.astype(np.float64) - ref)) / max(np.max(np.abs(ref)), 1e-300))


SMALL = [
    # f, fo, n, k      (several tiles, ragged tails, anisotropic, 2D, k = n, k = 1)
    (1, 4, (16, 16, 16), (3, 3, 3)),
    (3, 5, (9, 10, 11), (2, 3, 4)),
    (5, 3, (1, 20, 23), (1, 5, 4)),
    (40, 40, (12, 12, 14), (3, 3, 3)),
    (2, 2, (4, 4, 4), (4, 4, 4)),
    (3, 2, (6, 7, 8), (1, 1, 1)),
    (7, 9, (17, 13, 20), (5, 3, 2)),
    (4, 6, (7, 25, 15), (3, 1, 5)),
    (17, 33, (8, 9, 35), (2, 2, 3)),
    (9, 130, (6, 7, 8), (2, 2, 2)),       # more than 128 output maps: several map groups
    (131, 5, (5, 6, 9), (2, 1, 3)),
    (3, 4, (81, 50, 36), (3, 4, 2)),      # three different transform extents, all register-resident passes
    (2, 3, (40, 100, 30), (2, 3, 3)),     # y extent above 96: LDS pass between two register passes
    (1, 2, (3, 128, 256), (2, 5, 3)),     # long pencils: radix-16 and radix-8 LDS passes (256 = 16 x 16, 128 = 16 x 8)
    (2, 1, (1, 192, 160), (1, 3, 3)),     # 192 = 16 x 4 x 3, 160 = 16 x 2 x 5
    (1, 1, (1, 120, 104), (1, 2, 2)),     # 120 = 8 x 3 x 5, 104 -> 108 = 4 x 3 x 3 x 3
    (2, 2, (1, 253, 20), (1, 4, 3)),      # y extent 256: two-level strided pass, zero-extended, ragged pencil chunk
    (1, 2, (256, 5, 6), (3, 2, 2)),       # z extent 256
]


@pytest.mark.parametrize("mode", ["direct", "fft"])
@pytest.mark.parametrize("f,fo,n,k", SMALL)
def test_three_passes_match_the_oracle(f, fo, n, k, mode):
    print("case", f, fo, n, k, mode, flush=True)
    cfg = synth.LayerShape("t", f, fo, n, k, 1.0, 77 + f + fo)
    inp, w, gout = synth.layer_tensors(cfg)
    p = znn.Plan(f, fo, n, k, mode)
    d_in, d_w, d_g = dev(inp), dev(w), dev(gout)
    out = host(p.fwd(d_in, d_w))
    gin = host(p.bwd(d_g, d_w))
    gw = host(p.wgrad(d_in, d_g))
    tol = TOL[mode]
    assert rel_err(out, oracle.conv3d_fwd(inp, w)) <= tol
    assert rel_err(gin, oracle.conv3d_bwd(gout, w, n)) <= tol
    assert rel_err(gw, oracle.conv3d_wgrad(inp, gout)) <= tol
    # run-to-run reproducibility: no atomics, fixed summation order
    assert np.array_equal(out, host(p.fwd(d_in, d_w)))
    assert np.array_equal(gin, host(p.bwd(d_g, d_w)))
    assert np.array_equal(gw, host(p.wgrad(d_in, d_g)))
    p.close()


DIRECT_TAPS = [
    # f, fo, n, k, s: shapes that steer the direct kernels through every way they walk the taps and
    # fetch the halo boxes (x-tap groups of 11, 7, 5, 4, 3, 2 and single taps; odd and even numbers of
    # groups; a last chunk of fewer than four input maps behind several full ones; input maps split
    # over workgroups with a ragged last share; boxes too wide for two halo buffers)
    (10, 7, (9, 9, 20), (2, 2, 7), (1, 1, 1)),
    (6, 5, (8, 9, 16), (3, 1, 6), (1, 1, 1)),
    (9, 4, (7, 8, 19), (1, 3, 9), (1, 1, 1)),
    (5, 6, (6, 7, 22), (2, 1, 10), (1, 1, 1)),
    (4, 3, (5, 6, 24), (1, 2, 11), (1, 1, 1)),
    (7, 8, (5, 8, 30), (2, 2, 14), (1, 1, 1)),
    (6, 5, (4, 7, 28), (1, 2, 13), (1, 1, 1)),
    (5, 9, (3, 14, 40), (1, 3, 22), (1, 1, 1)),
    (11, 5, (6, 6, 20), (1, 1, 8), (1, 1, 1)),
    (13, 6, (10, 10, 10), (3, 3, 2), (1, 1, 1)),
    (27, 40, (14, 14, 14), (3, 3, 3), (1, 1, 1)),
    (40, 3, (20, 20, 20), (3, 3, 3), (4, 4, 4)),
    (21, 24, (26, 26, 26), (3, 3, 3), (4, 4, 4)),
    (18, 40, (30, 30, 30), (5, 5, 5), (1, 1, 1)),
    # output-side map counts of the form 16 q + r, 1 <= r <= 8, in one or both directions: the last r
    # maps run as an 8-map block beside q full tiles (q = 1 .. 7), for every tap-group width, with a
    # ragged last chunk of input maps, split input maps, sparse taps and a 2D layer
    (10, 24, (9, 9, 20), (2, 2, 7), (1, 1, 1)),
    (22, 20, (8, 9, 16), (3, 1, 6), (1, 1, 1)),
    (19, 36, (6, 7, 22), (2, 1, 10), (1, 1, 1)),
    (24, 17, (5, 6, 24), (1, 2, 11), (1, 1, 1)),
    (36, 40, (7, 8, 19), (1, 3, 9), (1, 1, 1)),
    (20, 56, (10, 10, 12), (3, 3, 2), (1, 1, 1)),
    (88, 24, (1, 40, 44), (1, 5, 4), (1, 1, 1)),
    (120, 72, (6, 10, 12), (3, 3, 3), (1, 1, 1)),
    (104, 97, (5, 9, 9), (2, 2, 2), (1, 1, 1)),
    (23, 21, (14, 14, 14), (3, 3, 3), (2, 2, 2)),
    (33, 24, (6, 6, 10), (2, 2, 2), (1, 1, 1)),
    # kernel gradient: many columns (every wave owns columns of its own; ragged last column group and
    # waves without columns), rows of gout of length 2 modulo 4 staged without padding, both together
    (12, 20, (8, 10, 16), (3, 3, 3), (1, 1, 1)),
    (9, 7, (6, 12, 24), (2, 3, 7), (1, 1, 1)),
    (100, 18, (4, 6, 12), (1, 2, 3), (1, 1, 1)),
    (70, 33, (3, 9, 16), (2, 2, 7), (1, 1, 1)),
    (45, 50, (1, 12, 36), (1, 3, 11), (1, 1, 1)),
]


@pytest.mark.parametrize("f,fo,n,k,s", DIRECT_TAPS)
def test_direct_kernels_on_every_tap_walk_and_halo_mode(f, fo, n, k, s):
    print("case", f, fo, n, k, s, flush=True)
    cfg = synth.LayerShape("t", f, fo, n, k, 1.0, 300 + f + fo, s)
    inp, w, gout = synth.layer_tensors(cfg)
    p = znn.Plan(f, fo, n, k, "direct", s)
    d_in, d_w, d_g = dev(inp), dev(w), dev(gout)
    out, gin, gw = host(p.fwd(d_in, d_w)), host(p.bwd(d_g, d_w)), host(p.wgrad(d_in, d_g))
    assert rel_err(out, oracle.conv3d_fwd(inp, w, s)) <= TOL["direct"]
    assert rel_err(gin, oracle.conv3d_bwd(gout, w, n, s)) <= TOL["direct"]
    assert rel_err(gw, oracle.conv3d_wgrad(inp, gout, s)) <= TOL["direct"]
    # a second call on the same plan (LDS contents of an earlier launch must not matter)
    assert np.array_equal(out, host(p.fwd(d_in, d_w)))
    assert np.array_equal(gin, host(p.bwd(d_g, d_w)))
    p.close()


SPARSE = [
    # f, fo, n, k, s      (sparse convolution: taps s voxels apart, Section 2)
    (3, 5, (11, 12, 13), (2, 3, 2), (2, 2, 3)),
    (8, 6, (1, 30, 29), (1, 3, 4), (1, 4, 2)),
    (20, 18, (14, 13, 22), (3, 3, 3), (2, 2, 2)),
    (5, 4, (9, 17, 8), (3, 2, 1), (4, 1, 5)),
    (2, 3, (36, 35, 8), (17, 17, 2), (2, 2, 3)),     # more taps than the pruned transforms take
]


@pytest.mark.parametrize("mode", ["direct", "fft"])
@pytest.mark.parametrize("f,fo,n,k,s", SPARSE)
def test_sparse_convolution_matches_the_oracle(f, fo, n, k, s, mode):
    print("case", f, fo, n, k, s, mode, flush=True)
    cfg = synth.LayerShape("t", f, fo, n, k, 1.0, 55 + f, s)
    inp, w, gout = synth.layer_tensors(cfg)
    p = znn.Plan(f, fo, n, k, mode, s)
    assert p.o == oracle.out_extents(n, k, s)
    d_in, d_w, d_g = dev(inp), dev(w), dev(gout)
    tol = TOL[mode]
    assert rel_err(host(p.fwd(d_in, d_w)), oracle.conv3d_fwd(inp, w, s)) <= tol
    assert rel_err(host(p.bwd(d_g, d_w)), oracle.conv3d_bwd(gout, w, n, s)) <= tol
    assert rel_err(host(p.wgrad(d_in, d_g)), oracle.conv3d_wgrad(inp, gout, s)) <= tol
    p.close()


FOLDED = [
    # f, fo, n, k, s: FFT layers large enough for the multiply-accumulate that folds the kernel
    # transform's last axis in; N_z = 40 takes the one-base variant, N_z = 64 the four-base one
    (32, 32, (40, 40, 40), (3, 3, 3), (1, 1, 1)),
    (40, 36, (64, 40, 40), (3, 3, 3), (1, 2, 2)),
    (64, 64, (1, 256, 250), (1, 6, 3), (1, 1, 2)),
]


@pytest.mark.parametrize("f,fo,n,k,s", FOLDED)
def test_fft_layers_with_folded_kernel_transform_match_the_oracle(f, fo, n, k, s):
    print("case", f, fo, n, k, s, flush=True)
    cfg = synth.LayerShape("t", f, fo, n, k, 1.0 / np.sqrt(f * np.prod(k)), 91 + f, s)
    inp, w, gout = synth.layer_tensors(cfg)
    p = znn.Plan(f, fo, n, k, "fft", s)
    N = p.fft_extents
    full = f * fo * N[0] * N[1] * (N[2] // 2 + 1) * 8
    assert p.spectra_bytes() < full          # half spectra: the folded path is the one that runs
    d_in, d_w, d_g = dev(inp), dev(w), dev(gout)
    out = host(p.fwd(d_in, d_w))
    gin = host(p.bwd(d_g, d_w))
    assert rel_err(out, oracle.conv3d_fwd(inp, w, s)) <= TOL["fft"]
    assert rel_err(gin, oracle.conv3d_bwd(gout, w, n, s)) <= TOL["fft"]
    assert rel_err(host(p.wgrad(d_in, d_g)), oracle.conv3d_wgrad(inp, gout, s)) <= TOL["fft"]
    p.prepare_kernels(d_w)                   # resident half spectra give the same bits
    assert np.array_equal(out, host(p.fwd(d_in, None)))
    assert np.array_equal(gin, host(p.bwd(d_g, None)))
    p.close()


@pytest.mark.parametrize("f,fo,n,k", [(12, 10, (16, 20, 18), (3, 3, 3)), (9, 6, (1, 32, 30), (1, 5, 3)),
                                      (40, 40, (32, 32, 32), (5, 5, 5))])
def test_both_spectra_layouts_match_the_oracle_and_cannot_be_mixed(f, fo, n, k):
    """Full kernel spectra (Section 4: the memoized kernel transforms, streamed by the
    multiply-accumulate) and half spectra (last transform axis folded into the
    multiply-accumulate) on the same layer, each chosen through the ABI."""
    cfg = synth.LayerShape("t", f, fo, n, k, 1.0 / np.sqrt(f * np.prod(k)), 300 + f)
    inp, w, gout = synth.layer_tensors(cfg)
    d_in, d_w, d_g = dev(inp), dev(w), dev(gout)
    r_out, r_gin = oracle.conv3d_fwd(inp, w), oracle.conv3d_bwd(gout, w, n)
    p = znn.Plan(f, fo, n, k, "fft")
    N = p.fft_extents
    full = f * fo * N[0] * N[1] * (N[2] // 2 + 1) * 8
    sizes = {}
    for layout in ("full", "folded"):
        p.set_spectra_layout(layout)
        assert p.spectra_layout == layout
        sizes[layout] = p.spectra_bytes()
        assert rel_err(host(p.fwd(d_in, d_w)), r_out) <= TOL["fft"], layout
        assert rel_err(host(p.bwd(d_g, d_w)), r_gin) <= TOL["fft"], layout
        p.prepare_kernels(d_w)
        # the layout of attached spectra cannot be changed under them
        with pytest.raises(znn.ZnnError) as e:
            p.set_spectra_layout("full" if layout == "folded" else "folded")
        assert e.value.code == znn.ZNN_EINVAL and p.spectra_layout == layout
        assert rel_err(host(p.fwd(d_in, None)), r_out) <= TOL["fft"], layout
        assert rel_err(host(p.bwd(d_g, None)), r_gin) <= TOL["fft"], layout
        p.release_kernels()
    assert sizes["full"] == (full + 255) // 256 * 256 and sizes["folded"] < full
    p.close()


REG_EXTENTS = [8, 9, 10, 12, 15, 16, 18, 20, 24, 25, 27, 30, 32, 36, 40, 45, 48, 50, 54, 60, 64, 72, 75, 80, 81,
               90, 96]


@pytest.mark.parametrize("N", REG_EXTENTS)
def test_fft_passes_with_register_resident_pencils_for_every_extent(N):
    """Every extent the register-resident y / z passes are instantiated for, on both axes
    (the x axis always takes the LDS pass), plus 100 (> 96: LDS passes on all axes)."""
    print("case", N, flush=True)
    for n, k in (((N, 6, 7), (3, 2, 2)), ((4, N, 7), (2, 3, 2))):
        cfg = synth.LayerShape("t", 2, 3, n, k, 1.0, 200 + N)
        inp, w, gout = synth.layer_tensors(cfg)
        p = znn.Plan(2, 3, n, k, "fft")
        assert p.fft_extents[0 if n[0] == N else 1] == N
        d_in, d_w, d_g = dev(inp), dev(w), dev(gout)
        assert rel_err(host(p.fwd(d_in, d_w)), oracle.conv3d_fwd(inp, w)) <= TOL["fft"], (n, "fwd")
        assert rel_err(host(p.bwd(d_g, d_w)), oracle.conv3d_bwd(gout, w, n)) <= TOL["fft"], (n, "bwd")
        assert rel_err(host(p.wgrad(d_in, d_g)), oracle.conv3d_wgrad(inp, gout)) <= TOL["fft"], (n, "wgrad")
        p.close()


@pytest.mark.parametrize("N", [2 * h for h in REG_EXTENTS])
def test_fft_x_passes_with_register_resident_rows_for_every_extent(N):
    """Every transform length the one-row-per-thread x passes are instantiated for (N = 2 H), once with
    rows that fill the line and once zero-extended, with row counts that leave a ragged last wave."""
    print("case", N, flush=True)

    def next_smooth(n):
        while True:
            t = n
            for q in (2, 3, 5):
                while t % q == 0:
                    t //= q
            if t == 1:
                return n
            n += 1

    shorter = [nx for nx in range(N - 1, N - 8, -1) if next_smooth(nx) == N]
    for nx in [N] + shorter[-1:]:
        n, k = (5, 17, nx), (2, 3, 4)
        cfg = synth.LayerShape("t", 2, 3, n, k, 1.0, 500 + N)
        inp, w, gout = synth.layer_tensors(cfg)
        p = znn.Plan(2, 3, n, k, "fft")
        assert p.fft_extents[2] == N
        d_in, d_w, d_g = dev(inp), dev(w), dev(gout)
        assert rel_err(host(p.fwd(d_in, d_w)), oracle.conv3d_fwd(inp, w)) <= TOL["fft"], (n, "fwd")
        assert rel_err(host(p.bwd(d_g, d_w)), oracle.conv3d_bwd(gout, w, n)) <= TOL["fft"], (n, "bwd")
        assert rel_err(host(p.wgrad(d_in, d_g)), oracle.conv3d_wgrad(inp, gout)) <= TOL["fft"], (n, "wgrad")
        p.close()


@pytest.mark.parametrize("N", [16, 18, 20, 24, 30, 32, 36, 40, 48, 50, 54, 60, 64, 72, 80, 90, 96])
def test_fft_x_and_y_passes_in_one_launch_for_every_extent(N):
    """Equal x and y transform lengths take both passes in one launch (a plane per workgroup): every
    length it is instantiated for, with planes that fill the transform and with zero-extended ones
    (which also shifts the output gradient's embedding and the crops of the inverse)."""
    print("case", N, flush=True)

    def next_smooth(n):
        while True:
            t = n
            for q in (2, 3, 5):
                while t % q == 0:
                    t //= q
            if t == 1:
                return n
            n += 1

    shorter = [m for m in range(N - 1, N - 8, -1) if next_smooth(m) == N]
    cases = [(N, N)] + ([(shorter[-1], shorter[0])] if shorter else [])
    for ny, nx in cases:
        # kernels of a few short rows take a pass of their own (one wave per plane, up to 16 rows of 16 taps);
        # a kernel with more rows goes through the general pass like an image
        kernels = [(3, 2, 4), (2, min(16, ny - 2), min(16, nx - 3))] + ([(1, 17, 5)] if ny >= 20 else [])
        for k in kernels:
            n = (8, ny, nx)
            cfg = synth.LayerShape("t", 3, 2, n, k, 1.0, 600 + N)
            inp, w, gout = synth.layer_tensors(cfg)
            p = znn.Plan(3, 2, n, k, "fft")
            assert p.fft_extents[1:] == (N, N)
            d_in, d_w, d_g = dev(inp), dev(w), dev(gout)
            assert rel_err(host(p.fwd(d_in, d_w)), oracle.conv3d_fwd(inp, w)) <= TOL["fft"], (n, k, "fwd")
            assert rel_err(host(p.bwd(d_g, d_w)), oracle.conv3d_bwd(gout, w, n)) <= TOL["fft"], (n, k, "bwd")
            assert rel_err(host(p.wgrad(d_in, d_g)), oracle.conv3d_wgrad(inp, gout)) <= TOL["fft"], (n, k, "wgrad")
            if k[0] > 1 or p.spectra_layout == "folded":
                p.set_spectra_layout("folded" if p.spectra_layout == "full" else "full")    # the other kernel transform as well
                assert rel_err(host(p.fwd(d_in, d_w)), oracle.conv3d_fwd(inp, w)) <= TOL["fft"], (n, k, "fwd, other layout")
            p.close()


@pytest.mark.parametrize("N", [100, 108, 120, 128, 135, 144, 150, 160, 180, 192, 225, 240, 256])
def test_fft_strided_passes_in_two_levels_for_every_extent(N):
    """Strided passes of lengths above the register limit that split into two factors of at most 16 keep the
    samples in registers at both levels: every such length, along y (2D layer, ragged chunk of pencils) and
    along z (pencils a plane apart), zero-extended inputs and cropped outputs included."""
    print("case", N, flush=True)
    for f, fo, n, k in ((2, 1, (1, N, 10), (1, 4, 3)), (1, 2, (N - 1, 4, 6), (5, 2, 2))):
        cfg = synth.LayerShape("t", f, fo, n, k, 1.0, 800 + N)
        inp, w, gout = synth.layer_tensors(cfg)
        p = znn.Plan(f, fo, n, k, "fft")
        assert N in p.fft_extents
        d_in, d_w, d_g = dev(inp), dev(w), dev(gout)
        assert rel_err(host(p.fwd(d_in, d_w)), oracle.conv3d_fwd(inp, w)) <= TOL["fft"], (n, "fwd")
        assert rel_err(host(p.bwd(d_g, d_w)), oracle.conv3d_bwd(gout, w, n)) <= TOL["fft"], (n, "bwd")
        assert rel_err(host(p.wgrad(d_in, d_g)), oracle.conv3d_wgrad(inp, gout)) <= TOL["fft"], (n, "wgrad")
        p.close()


@pytest.mark.parametrize("f,fo,n,k", [
    (2, 24, (32, 12, 21), (3, 2, 4)),       # one group of eight base frequencies per wave
    (2, 24, (64, 70, 80), (3, 3, 3)),       # two groups per wave: forward pass
    (24, 2, (64, 70, 80), (4, 3, 2)),       # two groups per wave: backward pass
    (2, 24, (96, 70, 80), (5, 3, 3)),       # three groups per wave (the headline layer's shape class): forward
    (24, 2, (96, 75, 80), (7, 2, 3)),       # three groups per wave: backward, odd number of in-plane frequencies
])
def test_fft_multiply_accumulate_finishes_the_inverse_transform_along_z(f, fo, n, k):
    """3D layers whose folded multiply-accumulate owns the whole z axis per wave transform their sums back along
    z before storing them: no separate inverse pass along z is launched for that pass, cropped rows are left
    out, and the results still match the oracle."""
    print("case", f, fo, n, k, flush=True)
    cfg = synth.LayerShape("t", f, fo, n, k, 1.0, 640 + f + n[0])
    inp, w, gout = synth.layer_tensors(cfg)
    p = znn.Plan(f, fo, n, k, "fft")
    p.set_spectra_layout("folded")
    d_in, d_w, d_g = dev(inp), dev(w), dev(gout)
    znn.trace_enable(True)
    try:
        znn.trace_collect()
        out = host(p.fwd(d_in, d_w))
        names_fwd = [name for name, _ in znn.trace_collect()]
        gin = host(p.bwd(d_g, d_w))
        names_bwd = [name for name, _ in znn.trace_collect()]
    finally:
        znn.trace_enable(False)
    fused = names_fwd if fo >= f else names_bwd
    assert any(name.startswith("spectral mac") and "MFMA" in name for name in fused), fused
    # y and x extents differ in all these shapes: the one strided inverse pass left is the one along y
    assert sum(name.startswith("fft axis inverse") for name in fused) == 1, fused
    assert rel_err(out, oracle.conv3d_fwd(inp, w)) <= TOL["fft"]
    assert rel_err(gin, oracle.conv3d_bwd(gout, w, n)) <= TOL["fft"]
    p.close()


def test_resident_kernel_spectra_give_the_same_result():
    f, fo, n, k = 6, 5, (10, 12, 9), (3, 4, 2)
    cfg = synth.LayerShape("t", f, fo, n, k, 1.0, 91)
    inp, w, gout = synth.layer_tensors(cfg)
    p = znn.Plan(f, fo, n, k, "fft")
    d_in, d_w, d_g = dev(inp), dev(w), dev(gout)
    out0, gin0 = host(p.fwd(d_in, d_w)), host(p.bwd(d_g, d_w))
    big = p.workspace_bytes(znn.ZNN_PASS_FWD)
    p.prepare_kernels(d_w)
    assert p.workspace_bytes(znn.ZNN_PASS_FWD) < big
    out1, gin1 = host(p.fwd(d_in, None)), host(p.bwd(d_g, None))
    assert np.array_equal(out0, out1) and np.array_equal(gin0, gin1)
    assert rel_err(out1, oracle.conv3d_fwd(inp, w)) <= TOL["fft"]
    p.release_kernels()
    assert p.workspace_bytes(znn.ZNN_PASS_FWD) == big
    p.close()


def test_memoized_node_spectra_give_the_same_kernel_gradient():
    f, fo, n, k = 5, 7, (11, 9, 12), (3, 2, 4)
    cfg = synth.LayerShape("t", f, fo, n, k, 1.0, 93)
    inp, w, gout = synth.layer_tensors(cfg)
    p = znn.Plan(f, fo, n, k, "fft")
    d_in, d_w, d_g = dev(inp), dev(w), dev(gout)
    gw0 = host(p.wgrad(d_in, d_g))
    p.enable_memo()
    with pytest.raises(znn.ZnnError):
        p.wgrad_memo()                      # forward and backward have not run yet
    out, gin = host(p.fwd(d_in, d_w)), host(p.bwd(d_g, d_w))
    gw1 = host(p.wgrad_memo())
    assert np.array_equal(gw0, gw1)
    assert rel_err(gw1, oracle.conv3d_wgrad(inp, gout)) <= TOL["fft"]
    assert rel_err(out, oracle.conv3d_fwd(inp, w)) <= TOL["fft"]
    assert rel_err(gin, oracle.conv3d_bwd(gout, w, n)) <= TOL["fft"]
    # a later forward pass replaces its half of the memo
    inp2 = synth.uniform_pm1(94, 0, inp.shape)
    p.fwd(dev(inp2), d_w)
    assert rel_err(host(p.wgrad_memo()), oracle.conv3d_wgrad(inp2, gout)) <= TOL["fft"]
    p.disable_memo()
    with pytest.raises(znn.ZnnError):
        p.wgrad_memo()
    p.close()


FILTERS = [((5, 6, 7), (2, 2, 2)), ((22, 22, 22), (2, 2, 2)), ((1, 30, 17), (1, 2, 2)),
           ((6, 5, 9), (3, 1, 4)), ((3, 3, 3), (3, 3, 3)), ((4, 5, 6), (1, 1, 1))]


@pytest.mark.parametrize("kind", ["random", "ties", "zeros"])
@pytest.mark.parametrize("n,win", FILTERS)
def test_maxfilter_is_exact_and_its_jacobian_matches(n, win, kind):
    print("case", n, win, kind, flush=True)
    maps = 5
    if kind == "random":
        x = synth.uniform_pm1(5, 0, (maps,) + n)
    elif kind == "ties":       # what a rectified image looks like: many exact zeros and repeats
        x = np.maximum(np.round(synth.uniform_pm1(6, 0, (maps,) + n) * 2), 0).astype(np.float32)
        x[0].flat[::3] = -0.0
    else:
        x = np.zeros((maps,) + n, dtype=np.float32)
    ref_out, ref_idx = oracle.maxfilter3d_fwd(x, win)
    out, idx = znn.maxfilter3d_fwd(dev(x), win)
    out, idx_h = host(out), host(idx)
    assert np.array_equal(out.astype(np.float64), ref_out)
    assert np.array_equal(idx_h, ref_idx)
    g = synth.uniform_pm1(7, 2, ref_out.shape)
    gin = host(znn.maxfilter3d_bwd(dev(g), idx, n, win))
    ref_gin = oracle.maxfilter3d_bwd(g, ref_idx, n, win)
    assert rel_err(gin, ref_gin) <= 1e-6


SPARSE_FILTERS = [((9, 8, 10), (2, 2, 2), (2, 2, 2)), ((7, 9, 6), (2, 3, 1), (3, 2, 4)),
                  ((1, 30, 17), (1, 2, 3), (1, 4, 2)), ((30, 30, 30), (2, 2, 2), (4, 4, 4))]


@pytest.mark.parametrize("kind", ["random", "ties"])
@pytest.mark.parametrize("n,win,s", SPARSE_FILTERS)
def test_sparse_maxfilter_is_exact_and_its_jacobian_matches(n, win, s, kind):
    print("case", n, win, s, kind, flush=True)
    maps = 4
    x = synth.uniform_pm1(15, 0, (maps,) + n)
    if kind == "ties":
        x = np.maximum(np.round(x * 2), 0).astype(np.float32)
    ref_out, ref_idx = oracle.maxfilter3d_fwd(x, win, s)
    out, idx = znn.maxfilter3d_fwd(dev(x), win, s)
    assert np.array_equal(host(out).astype(np.float64), ref_out)
    assert np.array_equal(host(idx), ref_idx)
    g = synth.uniform_pm1(16, 2, ref_out.shape)
    gin = host(znn.maxfilter3d_bwd(dev(g), idx, n, win, s))
    assert rel_err(gin, oracle.maxfilter3d_bwd(g, ref_idx, n, win, s)) <= 1e-6


POOLS = [((4, 6, 8), (2, 2, 2)), ((6, 3, 4), (3, 1, 2)), ((1, 32, 27), (1, 4, 3)), ((2, 2, 2), (2, 2, 2)),
         ((3, 4, 5), (1, 1, 1)), ((24, 26, 22), (2, 2, 2))]


@pytest.mark.parametrize("kind", ["random", "ties"])
@pytest.mark.parametrize("n,p", POOLS)
def test_maxpool_is_exact_and_its_jacobian_matches(n, p, kind):
    print("case", n, p, kind, flush=True)
    maps = 5
    x = synth.uniform_pm1(17, 0, (maps,) + n)
    if kind == "ties":
        x = np.maximum(np.round(x * 2), 0).astype(np.float32)
        x[0].flat[::3] = -0.0
    ref_out, ref_idx = oracle.maxpool3d_fwd(x, p)
    out, idx = znn.maxpool3d_fwd(dev(x), p)
    assert np.array_equal(host(out).astype(np.float64), ref_out)
    assert np.array_equal(host(idx), ref_idx)
    g = synth.uniform_pm1(18, 2, ref_out.shape)
    gin = host(znn.maxpool3d_bwd(dev(g), idx, n, p))
    assert np.array_equal(gin.astype(np.float64), oracle.maxpool3d_bwd(g, ref_idx, n, p))


@pytest.mark.parametrize("fn", ["rectify", "logistic", "tanh"])
def test_transfer_functions_match_the_oracle(fn):
    maps = 6
    x = synth.uniform_pm1(19, 0, (maps, 9, 10, 11), 4.0)
    b = synth.uniform_pm1(19, 4, (maps,), 0.5)
    y = host(znn.transfer_fwd(dev(x), dev(b), fn))
    assert rel_err(y, oracle.transfer_fwd(x, b, fn)) <= 1e-6
    gy = synth.uniform_pm1(19, 2, x.shape)
    gx = host(znn.transfer_bwd(dev(gy), dev(y), fn))
    assert rel_err(gx, oracle.transfer_bwd(gy, y, fn)) <= 1e-6


def test_cross_entropy_loss_gradient_matches_the_oracle():
    y = (0.02 + 0.96 * synth.uniform_01(20, 0, (3, 7, 8, 9))).astype(np.float32)
    t = synth.uniform_01(20, 3, y.shape)
    g = host(znn.loss_grad(dev(y), dev(t), "cross_entropy"))
    assert rel_err(g, oracle.loss_grad(y, t, "cross_entropy")) <= 1e-6
    assert np.array_equal(host(znn.loss_grad(dev(y), dev(t), "square")), y - t)


def test_small_net_with_every_layer_kind_matches_the_oracle_round():
    """conv (dense and sparse), all three transfer functions, dense and sparse max-filter,
    max-pooling and the cross-entropy loss in one training round."""
    from oracle import net as onet
    from paper_1510_06706_amd import net as znet
    layers = [("conv", 2, 5, (2, 3, 2)), ("transfer", "tanh"), ("maxfilter", (2, 1, 2)),
              ("conv", 5, 4, (2, 2, 1), (2, 1, 2)), ("transfer",), ("maxfilter", (2, 2, 1), (2, 1, 2)),
              ("maxpool", (1, 2, 2)), ("conv", 4, 3, (1, 2, 2)), ("transfer", "logistic")]
    in_shape = (2, 10, 12, 14)
    x, target, params = synth.net_tensors(layers, in_shape, 31)
    for mode in ("direct", "fft"):
        net = znet.Net(layers, in_shape, params, mode)
        acts, aux, gout, grads = net.train_round(dev(x), dev(target), 1e-2, loss="cross_entropy")
        p64 = [None if p is None else {k: v.astype(np.float64) for k, v in p.items()} for p in params]
        loss, r_acts, r_aux, r_grads, r_new = onet.train_round(layers, p64, x, target, 1e-2, "cross_entropy")
        assert rel_err(host(acts[-1]), r_acts[-1]) <= TOL[mode]
        for l, a in enumerate(r_aux):
            if a is not None:
                assert np.array_equal(host(aux[l]), a), ("argmax", l)
        for l, g in enumerate(r_grads):
            if g is not None:
                for k in g:
                    assert rel_err(host(grads[l][k]), g[k]) <= TOL[mode], (mode, l, k)
                    assert rel_err(host(net.params[l][k]), r_new[l][k]) <= TOL[mode], (mode, l, k)


def test_pointwise_steps_of_a_training_round():
    maps, vox = 7, 1000
    x = synth.uniform_pm1(8, 0, (maps, 10, 10, 10))
    b = synth.uniform_pm1(8, 4, (maps,), 0.1)
    y = host(znn.transfer_fwd(dev(x), dev(b)))
    want = np.maximum(x + b[:, None, None, None], 0)
    assert np.array_equal(y, want)
    gy = synth.uniform_pm1(8, 2, x.shape)
    gx = host(znn.transfer_bwd(dev(gy), dev(y)))
    assert np.array_equal(gx, np.where(want > 0, gy, 0).astype(np.float32))
    gb = host(znn.bias_grad(dev(gy)))
    assert rel_err(gb, gy.astype(np.float64).reshape(maps, -1).sum(1)) <= 1e-5
    t = synth.uniform_01(8, 3, x.shape)
    assert np.array_equal(host(znn.square_loss_grad(dev(x), dev(t))), x - t)
    p = dev(x.copy())
    znn.sgd_update(p, dev(gy), 0.01)
    assert np.allclose(host(p), x - np.float32(0.01) * gy, rtol=0, atol=1e-7)


def test_autotuner_times_both_methods_and_caches_its_choice():
    f, fo, n, k = 8, 8, (20, 20, 20), (3, 3, 3)
    chosen, ms = znn.autotune(f, fo, n, k)
    assert chosen in (znn.ZNN_DIRECT, znn.ZNN_FFT)
    assert all(np.isfinite(v) and v > 0 for row in ms for v in row)
    assert chosen == (znn.ZNN_FFT if sum(ms[1]) < sum(ms[0]) else znn.ZNN_DIRECT)
    p = znn.Plan(f, fo, n, k, "auto")
    assert p.mode == chosen
    p.close()


def test_round_autotuner_respects_the_memory_budget():
    f, fo, n, k = 8, 8, (20, 20, 20), (3, 3, 3)
    chosen, ms, nbytes = znn.autotune_round(f, fo, n, k)
    assert all(np.isfinite(v) and v > 0 for v in ms.values())
    assert chosen == min(ms, key=ms.get)
    assert nbytes["fft_memo"] > nbytes["fft"] > nbytes["direct"] > 0
    p = znn.Plan(f, fo, n, k, "auto")
    assert p.mode == (znn.ZNN_DIRECT if chosen == "direct" else znn.ZNN_FFT)
    p.close()
    # a budget just below what memoization holds rules it out, and only it
    chosen2, ms2, _ = znn.autotune_round(f, fo, n, k, memory_budget=nbytes["fft_memo"] - 1)
    assert np.isinf(ms2["fft_memo"]) and np.isfinite(ms2["fft"]) and np.isfinite(ms2["direct"])
    assert chosen2 in ("direct", "fft") and chosen2 == min(ms2, key=ms2.get)
    chosen3, ms3, _ = znn.autotune_round(f, fo, n, k, memory_budget=nbytes["direct"])
    assert chosen3 == "direct" and np.isinf(ms3["fft"]) and np.isinf(ms3["fft_memo"])
    with pytest.raises(znn.ZnnError) as e:
        znn.autotune_round(f, fo, n, k, memory_budget=nbytes["direct"] - 1)
    assert e.value.code == znn.ZNN_EWORKSPACE


@pytest.mark.parametrize("mode", ["fft_memo", "tuned"])
def test_training_round_with_memoized_spectra_matches_the_oracle(mode):
    """Kernels transformed once per round and shared by forward and backward, node spectra
    kept for the kernel gradient (Section 4, memoization); two rounds, so that the kernel
    spectra are refreshed after the update."""
    from oracle import net as onet
    from paper_1510_06706_amd import net as znet
    layers = [("conv", 2, 6, (3, 3, 3)), ("transfer",), ("maxfilter", (2, 2, 2)),
              ("conv", 6, 5, (2, 3, 2), (2, 2, 2)), ("transfer", "tanh"),
              ("conv", 5, 3, (3, 1, 2)), ("transfer", "logistic")]
    in_shape = (2, 14, 15, 16)
    x, target, params = synth.net_tensors(layers, in_shape, 41)
    net = znet.Net(layers, in_shape, params, mode)
    if mode == "tuned":
        assert set(net.tuning) == {0, 3, 5}
        print("tuned strategies", {l: t[0] for l, t in net.tuning.items()}, flush=True)
    p64 = [None if p is None else {k: v.astype(np.float64) for k, v in p.items()} for p in params]
    for rnd in range(2):
        acts, aux, gout, grads = net.train_round(dev(x), dev(target), 0.05)
        loss, r_acts, r_aux, r_grads, p64 = onet.train_round(layers, p64, x, target, 0.05)
        assert rel_err(host(acts[-1]), r_acts[-1]) <= 1e-3, rnd
        for l, g in enumerate(r_grads):
            if g is not None:
                for k in g:
                    assert rel_err(host(grads[l][k]), g[k]) <= 1e-3, (rnd, l, k)
                    assert rel_err(host(net.params[l][k]), p64[l][k]) <= 1e-3, (rnd, l, k)
