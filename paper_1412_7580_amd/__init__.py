"""Thin Python binding of libfftconv.so (the C ABI declared in include/fftconv.h).

Argument marshalling only: torch is used for device memory and streams, every step of the
computation runs in the HIP kernels.  There is no CPU or PyTorch fallback: if the library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIBPATH = os.path.join(_HERE, "libfftconv.so")
_lib = None

SYMBOLS = [
    "fftconv_create", "fftconv_destroy", "fftconv_set_stream", "fftconv_status_string",
    "fftconv_workspace_bytes", "fft_conv_fprop", "fft_conv_bprop", "fft_conv_accgrad",
    "fft_r2c_1d", "fft_c2r_1d", "fft_r2c_2d", "fft_c2r_2d",
    "fftconv_set_profiling", "fftconv_last_kernel_ms", "fftconv_last_kernel_label",
    "fftconv_saved_bytes", "fftconv_backward_workspace_bytes", "fft_conv_fprop_save", "fft_conv_backward",
    "fftconv_tiled_workspace_bytes", "fftconv_tile_basis", "fftconv_layer_basis",
    "fft_conv_fprop_tiled", "fft_conv_bprop_tiled", "fft_conv_accgrad_tiled", "fftconv_autotune_basis",
    "fftconv_saved_bytes_tiled", "fftconv_backward_workspace_bytes_tiled",
    "fft_conv_fprop_save_tiled", "fft_conv_backward_tiled",
    "fftconv_weights_bytes", "fft_conv_transform_weights", "fft_conv_fprop_weights", "fft_conv_bprop_weights",
    "fft_conv_fprop_fused", "fft_conv_bprop_fused", "fft_conv_accgrad_fused",
    "fftconv_padded_workspace_bytes",
    "fft_conv_fprop_padded", "fft_conv_bprop_padded", "fft_conv_accgrad_padded",
    "fftconv_saved_bytes_padded", "fftconv_backward_workspace_bytes_padded",
    "fft_conv_fprop_save_padded", "fft_conv_backward_padded",
    "fftconv_static_scratch_bytes", "fft_conv_fprop_static", "fftconv_describe_plan",
]


class FFTConvError(RuntimeError):
    pass


def load_library():
    """dlopen libfftconv.so (building it first only if it does not exist) and set prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIBPATH):
        from . import build as _build
        _build.build(force=True)
    # torch ships its own HIP runtime; import it first so that the library binds to the same
    # runtime instance that owns the tensors and streams it is handed.
    import torch  # noqa: F401
    lib = ctypes.CDLL(_LIBPATH)
    vp, i, l, f, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_long, ctypes.c_float, ctypes.c_size_t
    lib.fftconv_create.argtypes = [ctypes.POINTER(vp), i]
    lib.fftconv_destroy.argtypes = [vp]
    lib.fftconv_set_stream.argtypes = [vp, vp]
    lib.fftconv_status_string.argtypes = [i]
    lib.fftconv_status_string.restype = ctypes.c_char_p
    lib.fftconv_workspace_bytes.argtypes = [i] * 8
    lib.fftconv_workspace_bytes.restype = sz
    lib.fft_conv_fprop.argtypes = [vp, vp, vp, vp] + [i] * 7 + [vp, sz]
    lib.fft_conv_bprop.argtypes = [vp, vp, vp, vp] + [i] * 7 + [vp, sz]
    lib.fft_conv_accgrad.argtypes = [vp, vp, vp, vp] + [i] * 7 + [f, i, vp, sz]
    lib.fft_r2c_1d.argtypes = [vp, vp, vp, l, i, i]
    lib.fft_c2r_1d.argtypes = [vp, vp, vp, l, i, i]
    lib.fft_r2c_2d.argtypes = [vp, vp, vp, l, i, i, i]
    lib.fft_c2r_2d.argtypes = [vp, vp, vp, l, i, i, i]
    lib.fftconv_set_profiling.argtypes = [vp, i]
    lib.fftconv_last_kernel_ms.argtypes = [vp, ctypes.POINTER(f), i, ctypes.POINTER(i)]
    lib.fftconv_last_kernel_label.argtypes = [vp, i]
    lib.fftconv_last_kernel_label.restype = ctypes.c_char_p
    lib.fftconv_saved_bytes.argtypes = [i] * 7
    lib.fftconv_saved_bytes.restype = sz
    lib.fftconv_backward_workspace_bytes.argtypes = [i] * 7
    lib.fftconv_backward_workspace_bytes.restype = sz
    lib.fft_conv_fprop_save.argtypes = [vp, vp, vp, vp] + [i] * 7 + [vp, sz, vp, sz]
    lib.fft_conv_backward.argtypes = [vp, vp, vp, vp] + [i] * 7 + [f, i, vp, sz, vp, sz]
    lib.fftconv_tiled_workspace_bytes.argtypes = [i] * 9
    lib.fftconv_tiled_workspace_bytes.restype = sz
    lib.fftconv_tile_basis.argtypes = [i] * 5
    lib.fftconv_layer_basis.argtypes = [i] * 6 + [ctypes.POINTER(ctypes.c_int)] * 2
    lib.fftconv_layer_basis.restype = i
    lib.fft_conv_fprop_tiled.argtypes = [vp, vp, vp, vp] + [i] * 8 + [vp, sz]
    lib.fft_conv_bprop_tiled.argtypes = [vp, vp, vp, vp] + [i] * 8 + [vp, sz]
    lib.fft_conv_accgrad_tiled.argtypes = [vp, vp, vp, vp] + [i] * 7 + [f, i, i, vp, sz]
    lib.fftconv_autotune_basis.argtypes = [vp] * 7 + [i] * 8 + [ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_float)]
    lib.fftconv_saved_bytes_tiled.argtypes = [i] * 8
    lib.fftconv_saved_bytes_tiled.restype = sz
    lib.fftconv_backward_workspace_bytes_tiled.argtypes = [i] * 8
    lib.fftconv_backward_workspace_bytes_tiled.restype = sz
    lib.fft_conv_fprop_save_tiled.argtypes = [vp, vp, vp, vp] + [i] * 8 + [vp, sz, vp, sz]
    lib.fft_conv_backward_tiled.argtypes = [vp, vp, vp, vp] + [i] * 8 + [f, i, vp, sz, vp, sz]
    lib.fftconv_weights_bytes.argtypes = [i] * 8
    lib.fftconv_weights_bytes.restype = sz
    lib.fft_conv_transform_weights.argtypes = [vp, vp, vp, sz] + [i] * 8
    lib.fft_conv_fprop_weights.argtypes = [vp, vp, vp, sz, vp] + [i] * 9 + [vp, sz]
    lib.fft_conv_bprop_weights.argtypes = [vp, vp, vp, sz, vp] + [i] * 9 + [vp, sz]
    lib.fft_conv_fprop_fused.argtypes = [vp, vp, vp, sz, vp] + [i] * 7
    lib.fft_conv_bprop_fused.argtypes = [vp, vp, vp, sz, vp] + [i] * 7
    lib.fft_conv_accgrad_fused.argtypes = [vp, vp, vp, vp] + [i] * 7 + [f, i]
    lib.fftconv_padded_workspace_bytes.argtypes = [i] * 10
    lib.fftconv_padded_workspace_bytes.restype = sz
    lib.fft_conv_fprop_padded.argtypes = [vp, vp, vp, vp] + [i] * 9 + [vp, sz]
    lib.fft_conv_bprop_padded.argtypes = [vp, vp, vp, vp] + [i] * 9 + [vp, sz]
    lib.fft_conv_accgrad_padded.argtypes = [vp, vp, vp, vp] + [i] * 9 + [f, i, vp, sz]
    lib.fftconv_saved_bytes_padded.argtypes = [i] * 9
    lib.fftconv_saved_bytes_padded.restype = sz
    lib.fftconv_backward_workspace_bytes_padded.argtypes = [i] * 9
    lib.fftconv_backward_workspace_bytes_padded.restype = sz
    lib.fft_conv_fprop_save_padded.argtypes = [vp, vp, vp, vp] + [i] * 9 + [vp, sz, vp, sz]
    lib.fft_conv_backward_padded.argtypes = [vp, vp, vp, vp] + [i] * 9 + [f, i, vp, sz, vp, sz]
    lib.fftconv_describe_plan.argtypes = [i] * 11 + [ctypes.POINTER(ctypes.c_long), i]
    lib.fftconv_describe_plan.restype = i
    lib.fftconv_static_scratch_bytes.argtypes = []
    lib.fftconv_static_scratch_bytes.restype = sz
    lib.fft_conv_fprop_static.argtypes = [vp, vp, vp, vp] + [i] * 7
    _lib = lib
    return lib


def _check(rc: int, what: str):
    if rc != 0:
        msg = load_library().fftconv_status_string(rc).decode()
        raise FFTConvError(f"{what}: {msg} (status {rc})")


def _dev_f32(t, name):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise FFTConvError(f"{name} must be a contiguous float32 tensor in device memory")
    return t.data_ptr()


FPROP, BPROP, ACCGRAD = 0, 1, 2

PLAN_FIELDS = ("Nr Nc tiled rect bins tile_log2 planesA planesB planesC hA wA hB wB hC wC M N K conjA conjB "
               "a_rs a_cs b_rs b_cs c_rs c_cs offA offB offC total bytesA").split()
VIEW_FIELDS = "view C nty ntx dy dx oy ox H W".split()


def describe_plan(pass_, S, f, fo, h, w, kh, kw, tile_n=-1, pad_h=0, pad_w=0):
    """fftconv_describe_plan as a dict (host only): the fields of PLAN_FIELDS, and "A", "B", "C":
    dicts of VIEW_FIELDS.  Raises FFTConvError for shapes the planner rejects."""
    lib = load_library()
    buf = (ctypes.c_long * 64)()
    n = int(lib.fftconv_describe_plan(pass_, S, f, fo, h, w, kh, kw, tile_n, pad_h, pad_w, buf, 64))
    if n < 0:
        _check(-n, "fftconv_describe_plan")
    vals = [int(buf[k]) for k in range(n)]
    out = dict(zip(PLAN_FIELDS, vals))
    at = len(PLAN_FIELDS)
    for name in "ABC":
        out[name] = dict(zip(VIEW_FIELDS, vals[at:at + len(VIEW_FIELDS)]))
        at += len(VIEW_FIELDS)
    return out


class Handle:
    """Owner of one fftconv_handle; the methods mirror the C entry points one to one."""

    def __init__(self, device: int = 0):
        import torch
        if not torch.cuda.is_available():
            raise FFTConvError("no GPU visible: the HIP library cannot run (there is no CPU fallback)")
        self._lib = load_library()
        self._h = ctypes.c_void_p()
        _check(self._lib.fftconv_create(ctypes.byref(self._h), device), "fftconv_create")
        self.device = device
        self._stream = 0               # a new handle runs on the null stream

    def close(self):
        if self._h:
            self._lib.fftconv_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _sync_stream(self):
        import torch
        s = torch.cuda.current_stream().cuda_stream
        if s != self._stream:          # the handle keeps its stream: tell it only about changes
            _check(self._lib.fftconv_set_stream(self._h, ctypes.c_void_p(s)), "fftconv_set_stream")
            self._stream = s

    def workspace_bytes(self, pass_, S, f, fo, h, w, kh, kw) -> int:
        return int(self._lib.fftconv_workspace_bytes(pass_, S, f, fo, h, w, kh, kw))

    def set_profiling(self, on: bool):
        _check(self._lib.fftconv_set_profiling(self._h, 1 if on else 0), "fftconv_set_profiling")

    def last_kernel_ms(self):
        buf = (ctypes.c_float * 8)()
        n = ctypes.c_int(0)
        _check(self._lib.fftconv_last_kernel_ms(self._h, buf, 8, ctypes.byref(n)), "fftconv_last_kernel_ms")
        return [float(buf[k]) for k in range(n.value)]

    def last_kernel_labels(self):
        """Names of the kernels whose times last_kernel_ms() returns, in the same order."""
        out = []
        for k in range(8):
            s = self._lib.fftconv_last_kernel_label(self._h, k)
            if not s:
                break
            out.append(s.decode())
        return out

    def saved_bytes(self, S, f, fo, h, w, kh, kw) -> int:
        return int(self._lib.fftconv_saved_bytes(S, f, fo, h, w, kh, kw))

    def backward_workspace_bytes(self, S, f, fo, h, w, kh, kw) -> int:
        return int(self._lib.fftconv_backward_workspace_bytes(S, f, fo, h, w, kh, kw))

    # ---- convolution passes -------------------------------------------------------------
    def fft_conv_fprop(self, x, wt, y=None, ws=None):
        import torch
        S, f, h, w = x.shape
        fo, f2, kh, kw = wt.shape
        if f2 != f:
            raise FFTConvError("x and wt disagree on the number of input planes")
        if y is None:
            y = torch.empty((S, fo, h - kh + 1, w - kw + 1), device=x.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_fprop(self._h, _dev_f32(x, "x"), _dev_f32(wt, "wt"), _dev_f32(y, "y"),
                                        S, f, fo, h, w, kh, kw, *self._ws(ws)), "fft_conv_fprop")
        return y

    def static_scratch_bytes(self) -> int:
        return int(self._lib.fftconv_static_scratch_bytes())

    def fft_conv_fprop_static(self, x, wt, y):
        """fft_conv_fprop on the library's static scratch array: no allocation, here or in the
        library (so y is required)."""
        S, f, h, w = x.shape
        fo, f2, kh, kw = wt.shape
        if f2 != f:
            raise FFTConvError("x and wt disagree on the number of input planes")
        self._sync_stream()
        _check(self._lib.fft_conv_fprop_static(self._h, _dev_f32(x, "x"), _dev_f32(wt, "wt"), _dev_f32(y, "y"),
                                               S, f, fo, h, w, kh, kw), "fft_conv_fprop_static")
        return y

    def fft_conv_fprop_save(self, x, wt, saved, y=None, ws=None):
        """fprop that also leaves the transforms of x and wt in `saved` (a float32 device tensor
        of at least saved_bytes() bytes) for fft_conv_backward."""
        import torch
        S, f, h, w = x.shape
        fo, f2, kh, kw = wt.shape
        if f2 != f:
            raise FFTConvError("x and wt disagree on the number of input planes")
        if y is None:
            y = torch.empty((S, fo, h - kh + 1, w - kw + 1), device=x.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_fprop_save(self._h, _dev_f32(x, "x"), _dev_f32(wt, "wt"), _dev_f32(y, "y"),
                                             S, f, fo, h, w, kh, kw, *self._ws(saved), *self._ws(ws)),
               "fft_conv_fprop_save")
        return y

    def fft_conv_backward(self, gy, saved, f, h, w, kh, kw, gx=None, gw=None, want_gx=True, want_gw=True,
                          scale=1.0, accumulate=False, ws=None):
        """bprop and accGrad of one layer from gy and the transforms saved by fft_conv_fprop_save."""
        import torch
        S, fo, oh, ow = gy.shape
        if oh != h - kh + 1 or ow != w - kw + 1:
            raise FFTConvError("gy and (h, w, kh, kw) disagree")
        if want_gx and gx is None:
            gx = torch.empty((S, f, h, w), device=gy.device, dtype=torch.float32)
        if want_gw and gw is None:
            if accumulate:
                raise FFTConvError("accumulate needs an existing gw")
            gw = torch.empty((fo, f, kh, kw), device=gy.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_backward(self._h, _dev_f32(gy, "gy"),
                                           _dev_f32(gx, "gx") if want_gx else None,
                                           _dev_f32(gw, "gw") if want_gw else None,
                                           S, f, fo, h, w, kh, kw, float(scale), 1 if accumulate else 0,
                                           *self._ws(saved), *self._ws(ws)), "fft_conv_backward")
        return gx, gw

    def fft_conv_bprop(self, gy, wt, h, w, gx=None, ws=None):
        import torch
        S, fo, oh, ow = gy.shape
        fo2, f, kh, kw = wt.shape
        if fo2 != fo or oh != h - kh + 1 or ow != w - kw + 1:
            raise FFTConvError("gy, wt and (h, w) disagree")
        if gx is None:
            gx = torch.empty((S, f, h, w), device=gy.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_bprop(self._h, _dev_f32(gy, "gy"), _dev_f32(wt, "wt"), _dev_f32(gx, "gx"),
                                        S, f, fo, h, w, kh, kw, *self._ws(ws)), "fft_conv_bprop")
        return gx

    def fft_conv_accgrad(self, x, gy, gw=None, scale=1.0, accumulate=False, ws=None):
        import torch
        S, f, h, w = x.shape
        S2, fo, oh, ow = gy.shape
        if S2 != S:
            raise FFTConvError("x and gy disagree on the minibatch size")
        kh, kw = h - oh + 1, w - ow + 1
        if gw is None:
            if accumulate:
                raise FFTConvError("accumulate needs an existing gw")
            gw = torch.empty((fo, f, kh, kw), device=x.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_accgrad(self._h, _dev_f32(x, "x"), _dev_f32(gy, "gy"), _dev_f32(gw, "gw"),
                                          S, f, fo, h, w, kh, kw, float(scale), 1 if accumulate else 0,
                                          *self._ws(ws)), "fft_conv_accgrad")
        return gw

    # ---- tiled passes ---------------------------------------------------------------------
    def tiled_workspace_bytes(self, pass_, S, f, fo, h, w, kh, kw, tile_n) -> int:
        return int(self._lib.fftconv_tiled_workspace_bytes(pass_, S, f, fo, h, w, kh, kw, tile_n))

    def tile_basis(self, h, w, kh, kw, tile_n) -> int:
        return int(self._lib.fftconv_tile_basis(h, w, kh, kw, tile_n))

    def layer_basis(self, h, w, kh, kw, pad_h=0, pad_w=0):
        """(rows, columns, tiled) of the basis the ordinary entry points use for a layer."""
        nr, nc = ctypes.c_int(0), ctypes.c_int(0)
        rc = int(self._lib.fftconv_layer_basis(h, w, kh, kw, pad_h, pad_w, ctypes.byref(nr), ctypes.byref(nc)))
        if rc < 0:
            _check(-rc, "fftconv_layer_basis")
        return nr.value, nc.value, bool(rc)

    def fft_conv_fprop_tiled(self, x, wt, tile_n, y=None, ws=None):
        import torch
        S, f, h, w = x.shape
        fo, f2, kh, kw = wt.shape
        if f2 != f:
            raise FFTConvError("x and wt disagree on the number of input planes")
        if y is None:
            y = torch.empty((S, fo, h - kh + 1, w - kw + 1), device=x.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_fprop_tiled(self._h, _dev_f32(x, "x"), _dev_f32(wt, "wt"), _dev_f32(y, "y"),
                                              S, f, fo, h, w, kh, kw, int(tile_n), *self._ws(ws)),
               "fft_conv_fprop_tiled")
        return y

    def fft_conv_bprop_tiled(self, gy, wt, h, w, tile_n, gx=None, ws=None):
        import torch
        S, fo, oh, ow = gy.shape
        fo2, f, kh, kw = wt.shape
        if fo2 != fo or oh != h - kh + 1 or ow != w - kw + 1:
            raise FFTConvError("gy, wt and (h, w) disagree")
        if gx is None:
            gx = torch.empty((S, f, h, w), device=gy.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_bprop_tiled(self._h, _dev_f32(gy, "gy"), _dev_f32(wt, "wt"), _dev_f32(gx, "gx"),
                                              S, f, fo, h, w, kh, kw, int(tile_n), *self._ws(ws)),
               "fft_conv_bprop_tiled")
        return gx

    def fft_conv_accgrad_tiled(self, x, gy, tile_n, gw=None, scale=1.0, accumulate=False, ws=None):
        import torch
        S, f, h, w = x.shape
        S2, fo, oh, ow = gy.shape
        if S2 != S:
            raise FFTConvError("x and gy disagree on the minibatch size")
        kh, kw = h - oh + 1, w - ow + 1
        if gw is None:
            if accumulate:
                raise FFTConvError("accumulate needs an existing gw")
            gw = torch.empty((fo, f, kh, kw), device=x.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_accgrad_tiled(self._h, _dev_f32(x, "x"), _dev_f32(gy, "gy"), _dev_f32(gw, "gw"),
                                                S, f, fo, h, w, kh, kw, float(scale), 1 if accumulate else 0,
                                                int(tile_n), *self._ws(ws)), "fft_conv_accgrad_tiled")
        return gw

    def autotune_basis(self, x, wt, gy, y=None, gx=None, gw=None, reps=3):
        """Times the three passes at every candidate basis; returns (basis, ms of the three passes)."""
        import torch
        S, f, h, w = x.shape
        fo, f2, kh, kw = wt.shape
        if f2 != f or tuple(gy.shape) != (S, fo, h - kh + 1, w - kw + 1):
            raise FFTConvError("x, wt and gy disagree on the layer's shape")
        y = torch.empty_like(gy) if y is None else y
        gx = torch.empty_like(x) if gx is None else gx
        gw = torch.empty_like(wt) if gw is None else gw
        basis, ms = ctypes.c_int(0), ctypes.c_float(0.0)
        self._sync_stream()
        _check(self._lib.fftconv_autotune_basis(self._h, _dev_f32(x, "x"), _dev_f32(wt, "wt"), _dev_f32(gy, "gy"),
                                                _dev_f32(y, "y"), _dev_f32(gx, "gx"), _dev_f32(gw, "gw"),
                                                S, f, fo, h, w, kh, kw, int(reps), ctypes.byref(basis), ctypes.byref(ms)),
               "fftconv_autotune_basis")
        return int(basis.value), float(ms.value)

    def saved_bytes_tiled(self, S, f, fo, h, w, kh, kw, tile_n) -> int:
        return int(self._lib.fftconv_saved_bytes_tiled(S, f, fo, h, w, kh, kw, tile_n))

    def backward_workspace_bytes_tiled(self, S, f, fo, h, w, kh, kw, tile_n) -> int:
        return int(self._lib.fftconv_backward_workspace_bytes_tiled(S, f, fo, h, w, kh, kw, tile_n))

    def fft_conv_fprop_save_tiled(self, x, wt, tile_n, saved, y=None, ws=None):
        import torch
        S, f, h, w = x.shape
        fo, f2, kh, kw = wt.shape
        if f2 != f:
            raise FFTConvError("x and wt disagree on the number of input planes")
        if y is None:
            y = torch.empty((S, fo, h - kh + 1, w - kw + 1), device=x.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_fprop_save_tiled(self._h, _dev_f32(x, "x"), _dev_f32(wt, "wt"), _dev_f32(y, "y"),
                                                   S, f, fo, h, w, kh, kw, int(tile_n), *self._ws(saved), *self._ws(ws)),
               "fft_conv_fprop_save_tiled")
        return y

    def fft_conv_backward_tiled(self, gy, saved, f, h, w, kh, kw, tile_n, gx=None, gw=None, want_gx=True,
                                want_gw=True, scale=1.0, accumulate=False, ws=None):
        import torch
        S, fo, oh, ow = gy.shape
        if oh != h - kh + 1 or ow != w - kw + 1:
            raise FFTConvError("gy and (h, w, kh, kw) disagree")
        if want_gx and gx is None:
            gx = torch.empty((S, f, h, w), device=gy.device, dtype=torch.float32)
        if want_gw and gw is None:
            if accumulate:
                raise FFTConvError("accumulate needs an existing gw")
            gw = torch.empty((fo, f, kh, kw), device=gy.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_backward_tiled(self._h, _dev_f32(gy, "gy"),
                                                 _dev_f32(gx, "gx") if want_gx else None,
                                                 _dev_f32(gw, "gw") if want_gw else None,
                                                 S, f, fo, h, w, kh, kw, int(tile_n), float(scale),
                                                 1 if accumulate else 0, *self._ws(saved), *self._ws(ws)),
               "fft_conv_backward_tiled")
        return gx, gw

    # ---- weights transformed ahead --------------------------------------------------------
    def weights_bytes(self, f, fo, h, w, kh, kw, pad_h=0, pad_w=0) -> int:
        return int(self._lib.fftconv_weights_bytes(f, fo, h, w, kh, kw, pad_h, pad_w))

    def fft_conv_transform_weights(self, wt, h, w, pad_h=0, pad_w=0, wf=None):
        """Transform of wt for layers of h x w images; returns the (float32 device) buffer."""
        import torch
        fo, f, kh, kw = wt.shape
        if wf is None:
            wf = torch.empty(self.weights_bytes(f, fo, h, w, kh, kw, pad_h, pad_w) // 4, device=wt.device,
                             dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_transform_weights(self._h, _dev_f32(wt, "wt"), *self._ws(wf), f, fo, h, w, kh, kw,
                                                    pad_h, pad_w), "fft_conv_transform_weights")
        return wf

    def fft_conv_fprop_weights(self, x, wf, fo, kh, kw, pad_h=0, pad_w=0, y=None, ws=None):
        import torch
        S, f, h, w = x.shape
        if y is None:
            y = torch.empty((S, fo, h + 2 * pad_h - kh + 1, w + 2 * pad_w - kw + 1), device=x.device,
                            dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_fprop_weights(self._h, _dev_f32(x, "x"), *self._ws(wf), _dev_f32(y, "y"),
                                                S, f, fo, h, w, kh, kw, pad_h, pad_w, *self._ws(ws)),
               "fft_conv_fprop_weights")
        return y

    def fft_conv_fprop_fused(self, x, wf, fo, kh, kw, y=None):
        """One-launch fprop of a small layer; raises FFTConvError("unsupported ...") for others."""
        import torch
        S, f, h, w = x.shape
        if y is None:
            y = torch.empty((S, fo, h - kh + 1, w - kw + 1), device=x.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_fprop_fused(self._h, _dev_f32(x, "x"), *self._ws(wf), _dev_f32(y, "y"),
                                              S, f, fo, h, w, kh, kw), "fft_conv_fprop_fused")
        return y

    def fft_conv_bprop_fused(self, gy, wf, f, h, w, kh, kw, gx=None):
        """One-launch bprop of a small layer; raises FFTConvError("unsupported ...") for others."""
        import torch
        S, fo, oh, ow = gy.shape
        if oh != h - kh + 1 or ow != w - kw + 1:
            raise FFTConvError("gy and (h, w, kh, kw) disagree")
        if gx is None:
            gx = torch.empty((S, f, h, w), device=gy.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_bprop_fused(self._h, _dev_f32(gy, "gy"), *self._ws(wf), _dev_f32(gx, "gx"),
                                              S, f, fo, h, w, kh, kw), "fft_conv_bprop_fused")
        return gx

    def fft_conv_accgrad_fused(self, x, gy, gw=None, scale=1.0, accumulate=False):
        """One-launch accGrad of a small layer; raises FFTConvError("unsupported ...") for others."""
        import torch
        S, f, h, w = x.shape
        S2, fo, oh, ow = gy.shape
        if S2 != S:
            raise FFTConvError("x and gy disagree on the minibatch size")
        kh, kw = h - oh + 1, w - ow + 1
        if gw is None:
            if accumulate:
                raise FFTConvError("accumulate needs an existing gw")
            gw = torch.empty((fo, f, kh, kw), device=x.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_accgrad_fused(self._h, _dev_f32(x, "x"), _dev_f32(gy, "gy"), _dev_f32(gw, "gw"),
                                                S, f, fo, h, w, kh, kw, float(scale), 1 if accumulate else 0),
               "fft_conv_accgrad_fused")
        return gw

    def fft_conv_bprop_weights(self, gy, wf, f, h, w, kh, kw, pad_h=0, pad_w=0, gx=None, ws=None):
        import torch
        S, fo, oh, ow = gy.shape
        if oh != h + 2 * pad_h - kh + 1 or ow != w + 2 * pad_w - kw + 1:
            raise FFTConvError("gy and (h, w, kh, kw, padding) disagree")
        if gx is None:
            gx = torch.empty((S, f, h, w), device=gy.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_bprop_weights(self._h, _dev_f32(gy, "gy"), *self._ws(wf), _dev_f32(gx, "gx"),
                                                S, f, fo, h, w, kh, kw, pad_h, pad_w, *self._ws(ws)),
               "fft_conv_bprop_weights")
        return gx

    # ---- zero-padded layers ---------------------------------------------------------------
    def padded_workspace_bytes(self, pass_, S, f, fo, h, w, kh, kw, pad_h, pad_w) -> int:
        return int(self._lib.fftconv_padded_workspace_bytes(pass_, S, f, fo, h, w, kh, kw, pad_h, pad_w))

    def fft_conv_fprop_padded(self, x, wt, pad_h, pad_w, y=None, ws=None):
        import torch
        S, f, h, w = x.shape
        fo, f2, kh, kw = wt.shape
        if f2 != f:
            raise FFTConvError("x and wt disagree on the number of input planes")
        if y is None:
            y = torch.empty((S, fo, h + 2 * pad_h - kh + 1, w + 2 * pad_w - kw + 1), device=x.device,
                            dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_fprop_padded(self._h, _dev_f32(x, "x"), _dev_f32(wt, "wt"), _dev_f32(y, "y"),
                                               S, f, fo, h, w, kh, kw, int(pad_h), int(pad_w), *self._ws(ws)),
               "fft_conv_fprop_padded")
        return y

    def fft_conv_bprop_padded(self, gy, wt, h, w, pad_h, pad_w, gx=None, ws=None):
        import torch
        S, fo, oh, ow = gy.shape
        fo2, f, kh, kw = wt.shape
        if fo2 != fo or oh != h + 2 * pad_h - kh + 1 or ow != w + 2 * pad_w - kw + 1:
            raise FFTConvError("gy, wt, (h, w) and the padding disagree")
        if gx is None:
            gx = torch.empty((S, f, h, w), device=gy.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_bprop_padded(self._h, _dev_f32(gy, "gy"), _dev_f32(wt, "wt"), _dev_f32(gx, "gx"),
                                               S, f, fo, h, w, kh, kw, int(pad_h), int(pad_w), *self._ws(ws)),
               "fft_conv_bprop_padded")
        return gx

    def fft_conv_accgrad_padded(self, x, gy, pad_h, pad_w, gw=None, scale=1.0, accumulate=False, ws=None):
        import torch
        S, f, h, w = x.shape
        S2, fo, oh, ow = gy.shape
        if S2 != S:
            raise FFTConvError("x and gy disagree on the minibatch size")
        kh, kw = h + 2 * pad_h - oh + 1, w + 2 * pad_w - ow + 1
        if gw is None:
            if accumulate:
                raise FFTConvError("accumulate needs an existing gw")
            gw = torch.empty((fo, f, kh, kw), device=x.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_accgrad_padded(self._h, _dev_f32(x, "x"), _dev_f32(gy, "gy"), _dev_f32(gw, "gw"),
                                                 S, f, fo, h, w, kh, kw, int(pad_h), int(pad_w), float(scale),
                                                 1 if accumulate else 0, *self._ws(ws)), "fft_conv_accgrad_padded")
        return gw

    def saved_bytes_padded(self, S, f, fo, h, w, kh, kw, pad_h, pad_w) -> int:
        return int(self._lib.fftconv_saved_bytes_padded(S, f, fo, h, w, kh, kw, pad_h, pad_w))

    def backward_workspace_bytes_padded(self, S, f, fo, h, w, kh, kw, pad_h, pad_w) -> int:
        return int(self._lib.fftconv_backward_workspace_bytes_padded(S, f, fo, h, w, kh, kw, pad_h, pad_w))

    def fft_conv_fprop_save_padded(self, x, wt, pad_h, pad_w, saved, y=None, ws=None):
        import torch
        S, f, h, w = x.shape
        fo, f2, kh, kw = wt.shape
        if f2 != f:
            raise FFTConvError("x and wt disagree on the number of input planes")
        if y is None:
            y = torch.empty((S, fo, h + 2 * pad_h - kh + 1, w + 2 * pad_w - kw + 1), device=x.device,
                            dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_fprop_save_padded(self._h, _dev_f32(x, "x"), _dev_f32(wt, "wt"), _dev_f32(y, "y"),
                                                    S, f, fo, h, w, kh, kw, int(pad_h), int(pad_w),
                                                    *self._ws(saved), *self._ws(ws)), "fft_conv_fprop_save_padded")
        return y

    def fft_conv_backward_padded(self, gy, saved, f, h, w, kh, kw, pad_h, pad_w, gx=None, gw=None,
                                 want_gx=True, want_gw=True, scale=1.0, accumulate=False, ws=None):
        import torch
        S, fo, oh, ow = gy.shape
        if oh != h + 2 * pad_h - kh + 1 or ow != w + 2 * pad_w - kw + 1:
            raise FFTConvError("gy, (h, w, kh, kw) and the padding disagree")
        if want_gx and gx is None:
            gx = torch.empty((S, f, h, w), device=gy.device, dtype=torch.float32)
        if want_gw and gw is None:
            if accumulate:
                raise FFTConvError("accumulate needs an existing gw")
            gw = torch.empty((fo, f, kh, kw), device=gy.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_conv_backward_padded(self._h, _dev_f32(gy, "gy"),
                                                  _dev_f32(gx, "gx") if want_gx else None,
                                                  _dev_f32(gw, "gw") if want_gw else None,
                                                  S, f, fo, h, w, kh, kw, int(pad_h), int(pad_w), float(scale),
                                                  1 if accumulate else 0, *self._ws(saved), *self._ws(ws)),
               "fft_conv_backward_padded")
        return gx, gw

    @staticmethod
    def _ws(ws):
        if ws is None:
            return ctypes.c_void_p(0), 0
        return ctypes.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size()

    # ---- stand-alone FFTs ---------------------------------------------------------------
    def fft_r2c_1d(self, x, n, out=None):
        import torch
        B, n_in = x.shape
        if out is None:
            out = torch.empty((B, n // 2 + 1, 2), device=x.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_r2c_1d(self._h, _dev_f32(x, "in"), _dev_f32(out, "out"), B, n_in, n), "fft_r2c_1d")
        return out

    def fft_c2r_1d(self, X, n, n_out, out=None):
        import torch
        B = X.shape[0]
        if tuple(X.shape[1:]) != (n // 2 + 1, 2):
            raise FFTConvError("in must be [B, n/2+1, 2]")
        if out is None:
            out = torch.empty((B, n_out), device=X.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_c2r_1d(self._h, _dev_f32(X, "in"), _dev_f32(out, "out"), B, n, n_out), "fft_c2r_1d")
        return out

    def fft_r2c_2d(self, x, n, out=None):
        import torch
        B, h_in, w_in = x.shape
        if out is None:
            out = torch.empty((B, n, n // 2 + 1, 2), device=x.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_r2c_2d(self._h, _dev_f32(x, "in"), _dev_f32(out, "out"), B, h_in, w_in, n), "fft_r2c_2d")
        return out

    def fft_c2r_2d(self, X, n, h_out, w_out, out=None):
        import torch
        B = X.shape[0]
        if tuple(X.shape[1:]) != (n, n // 2 + 1, 2):
            raise FFTConvError("in must be [B, n, n/2+1, 2]")
        if out is None:
            out = torch.empty((B, h_out, w_out), device=X.device, dtype=torch.float32)
        self._sync_stream()
        _check(self._lib.fft_c2r_2d(self._h, _dev_f32(X, "in"), _dev_f32(out, "out"), B, n, h_out, w_out), "fft_c2r_2d")
        return out
