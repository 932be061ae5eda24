"""Parity of the three passes with the oracle on a seeded sweep of random layer shapes, both methods.

The hand-picked shapes of test_gpu_parity.py aim at known code paths; this sweep is for the ones nobody
thought of: map counts around the tile sizes (16 q + r), anisotropic and sparse kernels, 2D layers, long
rows and columns (transform lengths up to 288: register passes, LDS passes of every radix), tiny outputs.
"""
import numpy as np
import pytest

import oracle
from paper_1510_06706_amd import binding as znn
from paper_1510_06706_amd import synth

pytestmark = pytest.mark.gpu

TOL = {"direct": 1e-4, "fft": 1e-3}
WIDTHS = [1, 3, 8, 17, 24, 33, 40, 56, 72, 88, 104, 120, 136]


def rel_err(got, ref):
    return float(np.max(np.abs(got.astype(np.float64) - ref)) / max(np.max(np.abs(ref)), 1e-300))


def random_shapes(seed, count, long_rows):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        two_d = rng.random() < 0.25
        k = [int(v) for v in rng.integers(1, 8, 3)]
        s = [int(v) for v in rng.integers(1, 4, 3)] if rng.random() < 0.2 else [1, 1, 1]
        if two_d:
            k[0], s[0] = 1, 1
        if long_rows:
            extra = [int(rng.integers(0, 3)), int(rng.integers(0, 280)), int(rng.integers(0, 280))]
            f, fo = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        else:
            big = rng.random() < 0.3
            extra = [int(rng.integers(0, 40 if (big and i > 0) else 14)) for i in range(3)]
            f = int(rng.choice(WIDTHS)) if rng.random() < 0.5 else int(rng.integers(1, 20))
            fo = int(rng.choice(WIDTHS)) if rng.random() < 0.5 else int(rng.integers(1, 20))
        n = [sp * (kk - 1) + 1 + e for kk, sp, e in zip(k, s, extra)]
        if two_d:
            n[0] = 1
        vol = n[0] * n[1] * n[2]
        if f * fo * vol * k[0] * k[1] * k[2] > 6e8 or vol > 200000:
            continue
        out.append((f, fo, tuple(n), tuple(k), tuple(s)))
    return out


@pytest.mark.parametrize("long_rows", [False, True])
def test_random_layer_shapes_match_the_oracle(long_rows):
    import torch
    shapes = random_shapes(20151021 + int(long_rows), 250 if not long_rows else 120, long_rows)
    for it, (f, fo, n, k, s) in enumerate(shapes):
        cfg = synth.LayerShape("t", f, fo, n, k, 1.0, 7000 + it, s)
        inp, w, gout = synth.layer_tensors(cfg)
        refs = (oracle.conv3d_fwd(inp, w, s), oracle.conv3d_bwd(gout, w, n, s), oracle.conv3d_wgrad(inp, gout, s))
        d_in, d_w, d_g = (torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0") for a in (inp, w, gout))
        for mode in ("direct", "fft"):
            print("case", it, mode, f, fo, n, k, s, flush=True)
            p = znn.Plan(f, fo, n, k, mode, s)
            got = (p.fwd(d_in, d_w), p.bwd(d_g, d_w), p.wgrad(d_in, d_g))
            torch.cuda.synchronize()
            for name, g, r in zip(("fwd", "bwd", "wgrad"), got, refs):
                assert rel_err(g.cpu().numpy(), r) <= TOL[mode], (mode, name, f, fo, n, k, s)
            p.close()
