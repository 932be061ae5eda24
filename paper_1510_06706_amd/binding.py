"""ctypes binding of libznn.so: same names as include/znn.h, argument marshalling only.

Tensors are torch CUDA tensors (device memory and streams come from torch);
every compute step runs inside the library.  There is no fallback: if the
library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libznn.so")

ZNN_OK, ZNN_EINVAL, ZNN_EUNSUPPORTED, ZNN_EWORKSPACE, ZNN_EHIP = 0, -1, -2, -3, -4
ZNN_DIRECT, ZNN_FFT, ZNN_AUTO = 0, 1, 2
ZNN_PASS_FWD, ZNN_PASS_BWD, ZNN_PASS_WGRAD = 0, 1, 2
MODES = {"direct": ZNN_DIRECT, "fft": ZNN_FFT, "auto": ZNN_AUTO}

EXPORTS = [
    "znn_plan_create", "znn_plan_destroy", "znn_plan_mode", "znn_plan_fft_extents",
    "znn_plan_workspace_bytes", "znn_plan_spectra_bytes", "znn_conv_prepare_kernels",
    "znn_conv_release_kernels", "znn_conv3d_fwd", "znn_conv3d_bwd", "znn_conv3d_wgrad",
    "znn_maxfilter3d_fwd", "znn_maxfilter3d_bwd", "znn_transfer_fwd", "znn_transfer_bwd",
    "znn_bias_grad", "znn_square_loss_grad", "znn_sgd_update", "znn_autotune_workspace_bytes",
    "znn_autotune", "znn_last_error", "znn_trace_enable", "znn_trace_collect",
    "znn_plan_memo_bytes", "znn_conv_set_memo", "znn_conv3d_wgrad_memo",
    "znn_maxfilter3d_sparse_fwd", "znn_maxfilter3d_sparse_bwd", "znn_maxpool3d_fwd", "znn_maxpool3d_bwd",
    "znn_transfer_fn_fwd", "znn_transfer_fn_bwd", "znn_cross_entropy_loss_grad",
    "znn_autotune_round_workspace_bytes", "znn_autotune_round", "znn_accumulate",
    "znn_plan_set_spectra_layout", "znn_plan_spectra_layout", "znn_conv3d_fwd_static",
]
STATIC_SCRATCH_BYTES = 32 * 1024 * 1024
SPECTRA_LAYOUTS = {"auto": 0, "full": 1, "folded": 2}
STRATEGIES = ("direct", "fft", "fft_memo")
TRANSFER_FNS = {"rectify": 0, "logistic": 1, "tanh": 2}


class Vec3(ctypes.Structure):
    _fields_ = [("z", ctypes.c_int32), ("y", ctypes.c_int32), ("x", ctypes.c_int32)]


class ConvDesc(ctypes.Structure):
    _fields_ = [("fan_in", ctypes.c_int32), ("fan_out", ctypes.c_int32), ("image", Vec3),
                ("kernel", Vec3), ("sparsity", Vec3), ("mode", ctypes.c_int32)]


class TraceRecord(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 56), ("ms", ctypes.c_float)]


class RoundReport(ctypes.Structure):
    _fields_ = [("ms", ctypes.c_float * 3), ("bytes", ctypes.c_uint64 * 3), ("chosen", ctypes.c_int32)]


class ZnnError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__("znn error %d: %s" % (code, message))
        self.code = code


_lib = None


def lib():
    """Loads libznn.so (raises if it is missing: there is no other compute path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libznn.so is not built: run `python -m paper_1510_06706_amd.build` "
                               "(or __graft_entry__.build()) first")
        # torch ships its own HIP runtime; load it first so that this library binds to
        # the same runtime instance (one process, one runtime) instead of a second copy.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, i32, i64 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int64
        L.znn_last_error.restype = ctypes.c_char_p
        L.znn_plan_create.argtypes = [ctypes.POINTER(ConvDesc), ctypes.POINTER(vp)]
        L.znn_plan_destroy.argtypes = [vp]
        L.znn_plan_destroy.restype = None
        L.znn_plan_mode.argtypes = [vp, ctypes.POINTER(i32)]
        L.znn_plan_fft_extents.argtypes = [vp, ctypes.POINTER(Vec3)]
        L.znn_plan_workspace_bytes.argtypes = [vp, i32, ctypes.POINTER(sz)]
        L.znn_plan_spectra_bytes.argtypes = [vp, ctypes.POINTER(sz)]
        L.znn_plan_set_spectra_layout.argtypes = [vp, i32]
        L.znn_plan_spectra_layout.argtypes = [vp, ctypes.POINTER(i32)]
        L.znn_conv_prepare_kernels.argtypes = [vp, vp, vp, sz, vp, sz, vp]
        L.znn_conv_release_kernels.argtypes = [vp]
        for name in ("znn_conv3d_fwd", "znn_conv3d_bwd", "znn_conv3d_wgrad"):
            getattr(L, name).argtypes = [vp, vp, vp, vp, vp, sz, vp]
        L.znn_conv3d_fwd_static.argtypes = [vp, vp, vp, vp, vp]
        L.znn_maxfilter3d_fwd.argtypes = [i32, Vec3, Vec3, vp, vp, vp, vp]
        L.znn_maxfilter3d_bwd.argtypes = [i32, Vec3, Vec3, vp, vp, vp, vp]
        L.znn_maxfilter3d_sparse_fwd.argtypes = [i32, Vec3, Vec3, Vec3, vp, vp, vp, vp]
        L.znn_maxfilter3d_sparse_bwd.argtypes = [i32, Vec3, Vec3, Vec3, vp, vp, vp, vp]
        L.znn_maxpool3d_fwd.argtypes = [i32, Vec3, Vec3, vp, vp, vp, vp]
        L.znn_maxpool3d_bwd.argtypes = [i32, Vec3, Vec3, vp, vp, vp, vp]
        L.znn_transfer_fn_fwd.argtypes = [i32, i32, i64, vp, vp, vp, vp]
        L.znn_transfer_fn_bwd.argtypes = [i32, i32, i64, vp, vp, vp, vp]
        L.znn_cross_entropy_loss_grad.argtypes = [i64, vp, vp, vp, vp]
        L.znn_transfer_fwd.argtypes = [i32, i64, vp, vp, vp, vp]
        L.znn_transfer_bwd.argtypes = [i32, i64, vp, vp, vp, vp]
        L.znn_bias_grad.argtypes = [i32, i64, vp, vp, vp]
        L.znn_square_loss_grad.argtypes = [i64, vp, vp, vp, vp]
        L.znn_accumulate.argtypes = [i64, vp, vp, vp]
        L.znn_sgd_update.argtypes = [i64, ctypes.c_float, vp, vp, vp]
        L.znn_autotune_workspace_bytes.argtypes = [ctypes.POINTER(ConvDesc), ctypes.POINTER(sz)]
        L.znn_autotune.argtypes = [ctypes.POINTER(ConvDesc), vp, sz, vp, ctypes.POINTER(i32),
                                   ctypes.POINTER(ctypes.c_float * 3 * 2)]
        L.znn_autotune_round_workspace_bytes.argtypes = [ctypes.POINTER(ConvDesc), ctypes.POINTER(sz)]
        L.znn_autotune_round.argtypes = [ctypes.POINTER(ConvDesc), ctypes.c_uint64, vp, sz, vp,
                                         ctypes.POINTER(RoundReport)]
        L.znn_plan_memo_bytes.argtypes = [vp, ctypes.POINTER(sz)]
        L.znn_conv_set_memo.argtypes = [vp, vp, sz]
        L.znn_conv3d_wgrad_memo.argtypes = [vp, vp, vp, sz, vp]
        L.znn_trace_enable.argtypes = [i32]
        L.znn_trace_collect.argtypes = [ctypes.POINTER(TraceRecord), i32, ctypes.POINTER(i32)]
        for name in EXPORTS:
            if name not in ("znn_last_error", "znn_plan_destroy"):
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def last_error() -> str:
    return lib().znn_last_error().decode()


def _check(rc: int):
    if rc != ZNN_OK:
        raise ZnnError(rc, last_error())


def _v3(t: Sequence[int]) -> Vec3:
    return Vec3(int(t[0]), int(t[1]), int(t[2]))


def make_desc(fan_in, fan_out, image, kernel, mode="direct", sparsity=(1, 1, 1)) -> ConvDesc:
    m = MODES[mode] if isinstance(mode, str) else int(mode)
    return ConvDesc(int(fan_in), int(fan_out), _v3(image), _v3(kernel), _v3(sparsity), m)


def _stream_ptr(stream=None):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _ptr(t, dtype=None):
    """Device pointer of a contiguous CUDA tensor (None -> NULL)."""
    if t is None:
        return ctypes.c_void_p(0)
    import torch
    if not t.is_cuda:
        raise ValueError("tensor must live on the GPU")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError("tensor must be %s, got %s" % (dtype, t.dtype))
    return ctypes.c_void_p(t.data_ptr())


class Plan:
    """Owner of a znn_plan; methods mirror the C entry points."""

    def __init__(self, fan_in, fan_out, image, kernel, mode="direct", sparsity=(1, 1, 1)):
        self.desc = make_desc(fan_in, fan_out, image, kernel, mode, sparsity)
        self.f, self.fo = int(fan_in), int(fan_out)
        self.n, self.k = tuple(int(v) for v in image), tuple(int(v) for v in kernel)
        self.s = tuple(int(v) for v in sparsity)
        self.o = tuple(n - s * (k - 1) for n, k, s in zip(self.n, self.k, self.s))
        self._h = ctypes.c_void_p(0)
        self._ws = None
        self._spectra = None
        _check(lib().znn_plan_create(ctypes.byref(self.desc), ctypes.byref(self._h)))

    def close(self):
        if self._h:
            lib().znn_plan_destroy(self._h)
            self._h = ctypes.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def mode(self) -> int:
        m = ctypes.c_int32(-1)
        _check(lib().znn_plan_mode(self._h, ctypes.byref(m)))
        return m.value

    @property
    def fft_extents(self) -> Tuple[int, int, int]:
        v = Vec3()
        _check(lib().znn_plan_fft_extents(self._h, ctypes.byref(v)))
        return (v.z, v.y, v.x)

    def workspace_bytes(self, which: int) -> int:
        b = ctypes.c_size_t(0)
        _check(lib().znn_plan_workspace_bytes(self._h, which, ctypes.byref(b)))
        return b.value

    def spectra_bytes(self) -> int:
        b = ctypes.c_size_t(0)
        _check(lib().znn_plan_spectra_bytes(self._h, ctypes.byref(b)))
        return b.value

    def set_spectra_layout(self, layout: str):
        """'auto', 'full' (the kernel transforms themselves) or 'folded' (half spectra)."""
        _check(lib().znn_plan_set_spectra_layout(self._h, SPECTRA_LAYOUTS[layout]))

    @property
    def spectra_layout(self) -> str:
        v = ctypes.c_int32(-1)
        _check(lib().znn_plan_spectra_layout(self._h, ctypes.byref(v)))
        return {1: "full", 2: "folded"}[v.value]

    def _workspace(self, which: int, device):
        """Grows (never shrinks) a torch byte buffer used as the caller workspace."""
        import torch
        need = self.workspace_bytes(which)
        if need == 0:
            return ctypes.c_void_p(0), 0
        if self._ws is None or self._ws.numel() < need + 256:
            self._ws = None
            self._ws = torch.empty(need + 256, dtype=torch.uint8, device=device)
        base = self._ws.data_ptr()
        aligned = (base + 255) & ~255
        return ctypes.c_void_p(aligned), need

    def prepare_kernels(self, w, stream=None):
        """Transforms all kernels once; the spectra stay resident in a buffer this object owns."""
        import torch
        need = self.spectra_bytes()
        buf = getattr(self, "_spectra", None)
        if buf is None or buf.numel() != need + 256 or buf.device != w.device:
            buf = torch.empty(need + 256, dtype=torch.uint8, device=w.device)
        aligned = (buf.data_ptr() + 255) & ~255
        ws, wsb = self._workspace(ZNN_PASS_FWD, w.device)
        _check(lib().znn_conv_prepare_kernels(self._h, _ptr(w, torch.float32), ctypes.c_void_p(aligned), need,
                                              ws, wsb, _stream_ptr(stream)))
        self._spectra = buf

    def memo_bytes(self) -> int:
        b = ctypes.c_size_t(0)
        _check(lib().znn_plan_memo_bytes(self._h, ctypes.byref(b)))
        return b.value

    def enable_memo(self, device="cuda:0"):
        """Attaches a buffer (owned by this object) in which fwd / bwd leave their node spectra."""
        import torch
        need = self.memo_bytes()
        self._memo = torch.empty(need + 256, dtype=torch.uint8, device=device)
        aligned = (self._memo.data_ptr() + 255) & ~255
        _check(lib().znn_conv_set_memo(self._h, ctypes.c_void_p(aligned), need))

    def disable_memo(self):
        _check(lib().znn_conv_set_memo(self._h, ctypes.c_void_p(0), 0))
        self._memo = None

    def wgrad_memo(self, gw=None, device="cuda:0", stream=None):
        """Kernel gradient of the tensors given to the last fwd and bwd, from their memoized spectra."""
        import torch
        if gw is None:
            gw = torch.empty((self.fo, self.f) + self.k, dtype=torch.float32, device=device)
        assert tuple(gw.shape) == (self.fo, self.f) + self.k
        ws, wsb = self._workspace(ZNN_PASS_WGRAD, gw.device)
        _check(lib().znn_conv3d_wgrad_memo(self._h, _ptr(gw, torch.float32), ws, wsb, _stream_ptr(stream)))
        return gw

    def release_kernels(self):
        _check(lib().znn_conv_release_kernels(self._h))
        self._spectra = None

    def fwd(self, inp, w, out=None, stream=None):
        import torch
        assert tuple(inp.shape) == (self.f,) + self.n, inp.shape
        if w is not None:
            assert tuple(w.shape) == (self.fo, self.f) + self.k, w.shape
        if out is None:
            out = torch.empty((self.fo,) + self.o, dtype=torch.float32, device=inp.device)
        assert tuple(out.shape) == (self.fo,) + self.o
        ws, wsb = self._workspace(ZNN_PASS_FWD, inp.device)
        _check(lib().znn_conv3d_fwd(self._h, _ptr(inp, torch.float32), _ptr(w, torch.float32),
                                    _ptr(out, torch.float32), ws, wsb, _stream_ptr(stream)))
        return out

    def fwd_static(self, inp, w, out, stream=None):
        """znn_conv3d_fwd_static: the forward pass with the library's built-in scratch array; this
        wrapper allocates nothing either (the caller passes `out`)."""
        import torch
        assert tuple(inp.shape) == (self.f,) + self.n, inp.shape
        assert tuple(out.shape) == (self.fo,) + self.o
        _check(lib().znn_conv3d_fwd_static(self._h, _ptr(inp, torch.float32), _ptr(w, torch.float32),
                                           _ptr(out, torch.float32), _stream_ptr(stream)))
        return out

    def bwd(self, gout, w, gin=None, stream=None):
        import torch
        assert tuple(gout.shape) == (self.fo,) + self.o, gout.shape
        if w is not None:
            assert tuple(w.shape) == (self.fo, self.f) + self.k, w.shape
        if gin is None:
            gin = torch.empty((self.f,) + self.n, dtype=torch.float32, device=gout.device)
        assert tuple(gin.shape) == (self.f,) + self.n
        ws, wsb = self._workspace(ZNN_PASS_BWD, gout.device)
        _check(lib().znn_conv3d_bwd(self._h, _ptr(gout, torch.float32), _ptr(w, torch.float32),
                                    _ptr(gin, torch.float32), ws, wsb, _stream_ptr(stream)))
        return gin

    def wgrad(self, inp, gout, gw=None, stream=None):
        import torch
        assert tuple(inp.shape) == (self.f,) + self.n, inp.shape
        assert tuple(gout.shape) == (self.fo,) + self.o, gout.shape
        if gw is None:
            gw = torch.empty((self.fo, self.f) + self.k, dtype=torch.float32, device=inp.device)
        assert tuple(gw.shape) == (self.fo, self.f) + self.k
        ws, wsb = self._workspace(ZNN_PASS_WGRAD, inp.device)
        _check(lib().znn_conv3d_wgrad(self._h, _ptr(inp, torch.float32), _ptr(gout, torch.float32),
                                      _ptr(gw, torch.float32), ws, wsb, _stream_ptr(stream)))
        return gw


def maxfilter3d_fwd(inp, win, sparsity=(1, 1, 1), stream=None):
    import torch
    maps, n = inp.shape[0], tuple(inp.shape[1:])
    o = tuple(a - s * (b - 1) for a, b, s in zip(n, win, sparsity))
    if min(o) < 1:
        o = (0, 0, 0)
    out = torch.empty((maps,) + o, dtype=torch.float32, device=inp.device)
    idx = torch.empty((maps,) + o, dtype=torch.int32, device=inp.device)
    if tuple(sparsity) == (1, 1, 1):
        _check(lib().znn_maxfilter3d_fwd(maps, _v3(n), _v3(win), _ptr(inp, torch.float32), _ptr(out), _ptr(idx),
                                         _stream_ptr(stream)))
    else:
        _check(lib().znn_maxfilter3d_sparse_fwd(maps, _v3(n), _v3(win), _v3(sparsity), _ptr(inp, torch.float32),
                                                _ptr(out), _ptr(idx), _stream_ptr(stream)))
    return out, idx


def maxfilter3d_bwd(gout, idx, n, win, sparsity=(1, 1, 1), stream=None):
    import torch
    maps = gout.shape[0]
    gin = torch.empty((maps,) + tuple(n), dtype=torch.float32, device=gout.device)
    if tuple(sparsity) == (1, 1, 1):
        _check(lib().znn_maxfilter3d_bwd(maps, _v3(n), _v3(win), _ptr(gout, torch.float32), _ptr(idx, torch.int32),
                                         _ptr(gin), _stream_ptr(stream)))
    else:
        _check(lib().znn_maxfilter3d_sparse_bwd(maps, _v3(n), _v3(win), _v3(sparsity), _ptr(gout, torch.float32),
                                                _ptr(idx, torch.int32), _ptr(gin), _stream_ptr(stream)))
    return gin


def maxpool3d_fwd(inp, p, stream=None):
    import torch
    maps, n = inp.shape[0], tuple(inp.shape[1:])
    o = tuple(a // b if b > 0 else 0 for a, b in zip(n, p))
    out = torch.empty((maps,) + o, dtype=torch.float32, device=inp.device)
    idx = torch.empty((maps,) + o, dtype=torch.int32, device=inp.device)
    _check(lib().znn_maxpool3d_fwd(maps, _v3(n), _v3(p), _ptr(inp, torch.float32), _ptr(out), _ptr(idx),
                                   _stream_ptr(stream)))
    return out, idx


def maxpool3d_bwd(gout, idx, n, p, stream=None):
    import torch
    maps = gout.shape[0]
    gin = torch.empty((maps,) + tuple(n), dtype=torch.float32, device=gout.device)
    _check(lib().znn_maxpool3d_bwd(maps, _v3(n), _v3(p), _ptr(gout, torch.float32), _ptr(idx, torch.int32),
                                   _ptr(gin), _stream_ptr(stream)))
    return gin


def transfer_fwd(x, bias, fn="rectify", stream=None):
    import torch
    y = torch.empty_like(x)
    maps = x.shape[0]
    if fn == "rectify":
        _check(lib().znn_transfer_fwd(maps, x.numel() // maps, _ptr(x, torch.float32), _ptr(bias, torch.float32),
                                      _ptr(y), _stream_ptr(stream)))
    else:
        _check(lib().znn_transfer_fn_fwd(TRANSFER_FNS[fn], maps, x.numel() // maps, _ptr(x, torch.float32),
                                         _ptr(bias, torch.float32), _ptr(y), _stream_ptr(stream)))
    return y


def transfer_bwd(gy, y, fn="rectify", stream=None):
    import torch
    gx = torch.empty_like(gy)
    maps = gy.shape[0]
    if fn == "rectify":
        _check(lib().znn_transfer_bwd(maps, gy.numel() // maps, _ptr(gy, torch.float32), _ptr(y, torch.float32),
                                      _ptr(gx), _stream_ptr(stream)))
    else:
        _check(lib().znn_transfer_fn_bwd(TRANSFER_FNS[fn], maps, gy.numel() // maps, _ptr(gy, torch.float32),
                                         _ptr(y, torch.float32), _ptr(gx), _stream_ptr(stream)))
    return gx


def bias_grad(g, stream=None):
    import torch
    maps = g.shape[0]
    gb = torch.empty((maps,), dtype=torch.float32, device=g.device)
    _check(lib().znn_bias_grad(maps, g.numel() // maps, _ptr(g, torch.float32), _ptr(gb), _stream_ptr(stream)))
    return gb


def square_loss_grad(out, target, stream=None):
    import torch
    g = torch.empty_like(out)
    _check(lib().znn_square_loss_grad(out.numel(), _ptr(out, torch.float32), _ptr(target, torch.float32),
                                      _ptr(g), _stream_ptr(stream)))
    return g


def cross_entropy_loss_grad(out, target, stream=None):
    import torch
    g = torch.empty_like(out)
    _check(lib().znn_cross_entropy_loss_grad(out.numel(), _ptr(out, torch.float32), _ptr(target, torch.float32),
                                             _ptr(g), _stream_ptr(stream)))
    return g


def loss_grad(out, target, loss="square", stream=None):
    if loss == "square":
        return square_loss_grad(out, target, stream)
    if loss == "cross_entropy":
        return cross_entropy_loss_grad(out, target, stream)
    raise ValueError(loss)


def accumulate(y, x, stream=None):
    """y += x (node sum of a computation graph)."""
    import torch
    assert y.shape == x.shape
    _check(lib().znn_accumulate(y.numel(), _ptr(x, torch.float32), _ptr(y, torch.float32), _stream_ptr(stream)))
    return y


def sgd_update(p, g, eta, stream=None):
    import torch
    _check(lib().znn_sgd_update(p.numel(), float(eta), _ptr(g, torch.float32), _ptr(p, torch.float32),
                                _stream_ptr(stream)))
    return p


def autotune_workspace_bytes(desc: ConvDesc) -> int:
    b = ctypes.c_size_t(0)
    _check(lib().znn_autotune_workspace_bytes(ctypes.byref(desc), ctypes.byref(b)))
    return b.value


def autotune(fan_in, fan_out, image, kernel, device="cuda:0", stream=None, sparsity=(1, 1, 1)):
    """Returns (chosen mode, ms[method][pass]) and caches the choice for mode='auto' plans."""
    import torch
    desc = make_desc(fan_in, fan_out, image, kernel, "auto", sparsity)
    need = autotune_workspace_bytes(desc)
    buf = torch.empty(need + 256, dtype=torch.uint8, device=device)
    aligned = (buf.data_ptr() + 255) & ~255
    chosen = ctypes.c_int32(-1)
    ms = (ctypes.c_float * 3 * 2)()
    _check(lib().znn_autotune(ctypes.byref(desc), ctypes.c_void_p(aligned), need, _stream_ptr(stream),
                              ctypes.byref(chosen), ctypes.byref(ms)))
    return chosen.value, [[ms[m][p] for p in range(3)] for m in range(2)]


def autotune_round(fan_in, fan_out, image, kernel, memory_budget=None, sparsity=(1, 1, 1), device="cuda:0",
                   stream=None):
    """Times a whole training round of the layer as direct / FFT / FFT with memoized spectra,
    leaving out what exceeds ``memory_budget`` bytes (None = no limit).  Returns
    (chosen strategy name, {name: ms}, {name: bytes})."""
    import torch
    desc = make_desc(fan_in, fan_out, image, kernel, "auto", sparsity)
    b = ctypes.c_size_t(0)
    _check(lib().znn_autotune_round_workspace_bytes(ctypes.byref(desc), ctypes.byref(b)))
    budget = (1 << 62) if memory_budget is None else int(memory_budget)
    buf = torch.empty(b.value + 256, dtype=torch.uint8, device=device)
    aligned = (buf.data_ptr() + 255) & ~255
    rep = RoundReport()
    _check(lib().znn_autotune_round(ctypes.byref(desc), budget, ctypes.c_void_p(aligned), b.value,
                                    _stream_ptr(stream), ctypes.byref(rep)))
    return (STRATEGIES[rep.chosen], {n: float(rep.ms[i]) for i, n in enumerate(STRATEGIES)},
            {n: int(rep.bytes[i]) for i, n in enumerate(STRATEGIES)})


def trace_enable(on: bool):
    _check(lib().znn_trace_enable(1 if on else 0))


def trace_collect(capacity: int = 4096):
    """[(kernel role, ms)] of every launch recorded since the last call, in launch order."""
    buf = (TraceRecord * capacity)()
    n = ctypes.c_int32(0)
    _check(lib().znn_trace_collect(buf, capacity, ctypes.byref(n)))
    return [(buf[i].name.decode(), float(buf[i].ms)) for i in range(min(n.value, capacity))]
