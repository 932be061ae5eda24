"""CPU oracle for the ZNN convolutional-layer hot path (arXiv 1510.06706).

TEST INFRASTRUCTURE ONLY.  Only the test-suite, the smoke check and the
``cpu_baseline`` leg of the benchmark may import this package; the GPU library
never does, and nothing here imports the GPU library.

``znn_ref.c`` holds the plain double-precision definitions (nested loops);
this module is the ctypes binding around it plus numpy-level helpers.  All
functions take and return float64 numpy arrays (float32 inputs are widened
exactly).

Layouts: images ``[map, z, y, x]``; kernels ``[fan_out, fan_in, kz, ky, kx]``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "znn_ref.c")
_LIB = os.path.join(_HERE, "libznn_ref.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile znn_ref.c with gcc (-O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-o", tmp, _SRC]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.znn_ref_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().znn_ref_num_threads())


def _i3(v):
    a = (ctypes.c_int * 3)(*[int(t) for t in v])
    return a


def _d(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _check(rc, what):
    if rc != 0:
        raise ValueError("oracle %s rejected its arguments (rc=%d)" % (what, rc))


def out_extents(n, k, sparsity=(1, 1, 1)):
    """n' = n - s (k - 1) per axis (Section 2; s = 1 gives n - k + 1)."""
    return tuple(int(n[d]) - int(sparsity[d]) * (int(k[d]) - 1) for d in range(3))


def conv3d_fwd(inp, w, sparsity=(1, 1, 1)):
    """out[j] = sum_i valid_conv(in[i], w[j, i])   (Section 2, Convolution; optionally sparse)."""
    inp, w = _f64(inp), _f64(w)
    fo, f = w.shape[:2]
    assert inp.ndim == 4 and w.ndim == 5 and inp.shape[0] == f
    n, k = inp.shape[1:], w.shape[2:]
    o = out_extents(n, k, sparsity)
    if min(o) < 1:
        raise ValueError("oracle fwd rejected its arguments (kernel span exceeds the image)")
    out = np.empty((fo,) + o, dtype=np.float64)
    _check(_load().znn_ref_conv3d_fwd(f, fo, _i3(n), _i3(k), _i3(sparsity), _d(inp), _d(w), _d(out)), "fwd")
    return out


def conv3d_bwd(gout, w, n, sparsity=(1, 1, 1)):
    """gin[i] = sum_j full_conv(gout[j], reflect(w[j, i]))   (Section 3.1)."""
    gout, w = _f64(gout), _f64(w)
    fo, f = w.shape[:2]
    k = w.shape[2:]
    assert gout.shape == (fo,) + out_extents(n, k, sparsity)
    gin = np.empty((f,) + tuple(n), dtype=np.float64)
    _check(_load().znn_ref_conv3d_bwd(f, fo, _i3(n), _i3(k), _i3(sparsity), _d(gout), _d(w), _d(gin)), "bwd")
    return gin


def _kernel_extents(n, o, sparsity):
    k = []
    for d in range(3):
        span = int(n[d]) - int(o[d])
        assert span % int(sparsity[d]) == 0, "extents do not match the sparsity"
        k.append(span // int(sparsity[d]) + 1)
    return tuple(k)


def conv3d_wgrad(inp, gout, sparsity=(1, 1, 1)):
    """gw[j, i] = valid_conv(reflect(in[i]), gout[j])   (Section 3.2)."""
    inp, gout = _f64(inp), _f64(gout)
    f, fo = inp.shape[0], gout.shape[0]
    n = inp.shape[1:]
    k = _kernel_extents(n, gout.shape[1:], sparsity)
    gw = np.empty((fo, f) + k, dtype=np.float64)
    _check(_load().znn_ref_conv3d_wgrad(f, fo, _i3(n), _i3(k), _i3(sparsity), _d(inp), _d(gout), _d(gw)), "wgrad")
    return gw


def _at(fn, what, f, fo, n, k, a, b, pos, sparsity=(1, 1, 1)):
    pos = np.ascontiguousarray(np.asarray(pos, dtype=np.int64))
    val = np.empty(pos.shape, dtype=np.float64)
    rc = fn(f, fo, _i3(n), _i3(k), _i3(sparsity), _d(a), _d(b), ctypes.c_long(pos.size),
            pos.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), _d(val))
    _check(rc, what)
    return val


def conv3d_fwd_at(inp, w, pos, sparsity=(1, 1, 1)):
    """Forward outputs at flat positions ``pos`` of the [fo, n'] tensor."""
    inp, w = _f64(inp), _f64(w)
    fo, f = w.shape[:2]
    return _at(_load().znn_ref_conv3d_fwd_at, "fwd_at", f, fo, inp.shape[1:], w.shape[2:], inp, w, pos, sparsity)


def conv3d_bwd_at(gout, w, n, pos, sparsity=(1, 1, 1)):
    """Backward outputs at flat positions ``pos`` of the [f, n] tensor."""
    gout, w = _f64(gout), _f64(w)
    fo, f = w.shape[:2]
    return _at(_load().znn_ref_conv3d_bwd_at, "bwd_at", f, fo, n, w.shape[2:], gout, w, pos, sparsity)


def conv3d_wgrad_at(inp, gout, pos, sparsity=(1, 1, 1)):
    """Kernel-gradient entries at flat positions ``pos`` of the [fo, f, k] tensor."""
    inp, gout = _f64(inp), _f64(gout)
    f, fo = inp.shape[0], gout.shape[0]
    n = inp.shape[1:]
    k = _kernel_extents(n, gout.shape[1:], sparsity)
    return _at(_load().znn_ref_conv3d_wgrad_at, "wgrad_at", f, fo, n, k, inp, gout, pos, sparsity)


def _ip(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def maxfilter3d_fwd(inp, win, sparsity=(1, 1, 1)):
    """Sliding-window maximum and the flat input offset that supplied it (window taps
    ``sparsity`` voxels apart; output extents n - s (win - 1))."""
    inp = _f64(inp)
    maps, n = inp.shape[0], inp.shape[1:]
    o = out_extents(n, win, sparsity)
    if min(o) < 1:
        raise ValueError("oracle maxfilter_fwd rejected its arguments (window span exceeds the image)")
    out = np.empty((maps,) + o, dtype=np.float64)
    idx = np.empty((maps,) + o, dtype=np.int32)
    rc = _load().znn_ref_maxfilter3d_fwd(maps, _i3(n), _i3(win), _i3(sparsity), _d(inp), _d(out), _ip(idx))
    _check(rc, "maxfilter_fwd")
    return out, idx


def maxfilter3d_bwd(gout, idx, n, win, sparsity=(1, 1, 1)):
    """Max-filter Jacobian: scatter-add gout to the recorded argmax voxels."""
    gout = _f64(gout)
    idx = np.ascontiguousarray(np.asarray(idx, dtype=np.int32))
    maps = gout.shape[0]
    assert gout.shape[1:] == out_extents(n, win, sparsity) and idx.shape == gout.shape
    gin = np.empty((maps,) + tuple(n), dtype=np.float64)
    rc = _load().znn_ref_maxfilter3d_bwd(maps, _i3(n), _i3(win), _i3(sparsity), _d(gout), _ip(idx), _d(gin))
    _check(rc, "maxfilter_bwd")
    return gin


def maxpool3d_fwd(inp, p):
    """Block maximum over blocks of p voxels per axis and the flat input offset of each
    maximum (Section 2, Max-pooling); n must be divisible by p."""
    inp = _f64(inp)
    maps, n = inp.shape[0], inp.shape[1:]
    if any(int(n[d]) % int(p[d]) for d in range(3)):
        raise ValueError("oracle maxpool_fwd rejected its arguments (n not divisible by p)")
    o = tuple(int(n[d]) // int(p[d]) for d in range(3))
    out = np.empty((maps,) + o, dtype=np.float64)
    idx = np.empty((maps,) + o, dtype=np.int32)
    _check(_load().znn_ref_maxpool3d_fwd(maps, _i3(n), _i3(p), _d(inp), _d(out), _ip(idx)), "maxpool_fwd")
    return out, idx


def maxpool3d_bwd(gout, idx, n, p):
    """Max-pooling Jacobian (Section 3.1): every block is zero except at its forward maximum."""
    gout = _f64(gout)
    idx = np.ascontiguousarray(np.asarray(idx, dtype=np.int32))
    maps = gout.shape[0]
    assert idx.shape == gout.shape
    gin = np.empty((maps,) + tuple(n), dtype=np.float64)
    _check(_load().znn_ref_maxpool3d_bwd(maps, _i3(n), _i3(p), _d(gout), _ip(idx), _d(gin)), "maxpool_bwd")
    return gin


# ---------------------------------------------------------------- transfer functions and losses
# Section 2, "Transfer function": a bias is added to every voxel, then a nondecreasing
# nonlinearity is applied: the logistic function, the hyperbolic tangent or half-wave
# rectification.  The backward edge multiplies by the derivative, written through the
# forward output y (Section 3.1): rectifier 1 where y > 0 else 0; logistic y (1 - y);
# tanh 1 - y^2.
TRANSFER_FUNCTIONS = ("rectify", "logistic", "tanh")


def transfer_fwd(x, bias, fn="rectify"):
    v = _f64(x) + _f64(bias)[:, None, None, None]
    if fn == "rectify":
        return np.maximum(v, 0.0)
    if fn == "logistic":
        return 1.0 / (1.0 + np.exp(-v))
    if fn == "tanh":
        return np.tanh(v)
    raise ValueError(fn)


def transfer_bwd(gy, y, fn="rectify"):
    gy, y = _f64(gy), _f64(y)
    if fn == "rectify":
        return gy * (y > 0.0)
    if fn == "logistic":
        return gy * y * (1.0 - y)
    if fn == "tanh":
        return gy * (1.0 - y * y)
    raise ValueError(fn)


# Section 3: the loss compares actual and desired output; its gradient with respect to
# the actual output starts the backward pass.  The paper names the Euclidean distance and
# leaves the others open; the second loss here is the cross-entropy between a target in
# [0, 1] and an output in (0, 1) (the natural partner of a logistic output layer).
#   square:        L = 1/2 sum (y - t)^2                       dL/dy = y - t
#   cross-entropy: L = - sum t log y + (1 - t) log (1 - y)     dL/dy = (y - t) / (y (1 - y))
LOSSES = ("square", "cross_entropy")


def loss_value(y, t, loss="square"):
    y, t = _f64(y), _f64(t)
    if loss == "square":
        return 0.5 * float(np.sum((y - t) ** 2))
    if loss == "cross_entropy":
        return -float(np.sum(t * np.log(y) + (1.0 - t) * np.log(1.0 - y)))
    raise ValueError(loss)


def loss_grad(y, t, loss="square"):
    y, t = _f64(y), _f64(t)
    if loss == "square":
        return y - t
    if loss == "cross_entropy":
        return (y - t) / (y * (1.0 - y))
    raise ValueError(loss)
