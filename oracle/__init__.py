"""ctypes front-end of the fp64 CPU oracle (``oracle/oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by ``bench.py``'s ``cpu_baseline`` leg, never by the product package.  It
imports nothing from the HIP package.

Function names follow the paper's pass names (Section 2): fprop, bprop,
accGrad, plus the discrete Fourier transform of the Supplement.  All inputs
are converted to float64; all results are float64 numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc (plain -O3, no fast-math, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O3", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        lp = ctypes.POINTER(ctypes.c_long)
        i, l = ctypes.c_int, ctypes.c_long
        for name in ("oracle_conv_fprop", "oracle_conv_bprop", "oracle_conv_accgrad"):
            fn = getattr(lib, name)
            fn.argtypes = [dp, dp, dp, i, i, i, i, i, i, i, lp, l]
            fn.restype = None
        lib.oracle_dft_r2c_1d.argtypes = [dp, dp, l, i, i]
        lib.oracle_idft_c2r_1d.argtypes = [dp, dp, l, i, i]
        lib.oracle_dft_r2c_2d.argtypes = [dp, dp, l, i, i, i]
        lib.oracle_idft_c2r_2d.argtypes = [dp, dp, l, i, i, i]
        lib.oracle_dft2_bruteforce.argtypes = [dp, dp, i]
        lib.oracle_num_threads.restype = i
        _lib = lib
    return _lib


def _d(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _sel(sel):
    if sel is None:
        return None, None, 0
    s = np.ascontiguousarray(sel, dtype=np.int64)
    return s, s.ctypes.data_as(ctypes.POINTER(ctypes.c_long)), len(s)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def conv_fprop(x, w, sel=None):
    """y[S,f',oh,ow] (or [len(sel),oh,ow] for the output planes s*f'+j in sel)."""
    x, w = _d(x), _d(w)
    S, f, h, wd = x.shape
    fo, f2, kh, kw = w.shape
    assert f == f2 and kh <= h and kw <= wd
    oh, ow = h - kh + 1, wd - kw + 1
    keep, sp, ns = _sel(sel)
    y = np.empty((ns, oh, ow) if sel is not None else (S, fo, oh, ow))
    _load().oracle_conv_fprop(_p(x), _p(w), _p(y), S, f, fo, h, wd, kh, kw, sp, ns)
    return y


def conv_bprop(gy, w, h, wd, sel=None):
    """gx[S,f,h,w] (or the planes s*f+i in sel)."""
    gy, w = _d(gy), _d(w)
    S, fo, oh, ow = gy.shape
    fo2, f, kh, kw = w.shape
    assert fo == fo2 and oh == h - kh + 1 and ow == wd - kw + 1
    keep, sp, ns = _sel(sel)
    gx = np.empty((ns, h, wd) if sel is not None else (S, f, h, wd))
    _load().oracle_conv_bprop(_p(gy), _p(w), _p(gx), S, f, fo, h, wd, kh, kw, sp, ns)
    return gx


def conv_accgrad(x, gy, sel=None):
    """gw[f',f,kh,kw] (or the planes j*f+i in sel)."""
    x, gy = _d(x), _d(gy)
    S, f, h, wd = x.shape
    S2, fo, oh, ow = gy.shape
    assert S == S2
    kh, kw = h - oh + 1, wd - ow + 1
    keep, sp, ns = _sel(sel)
    gw = np.empty((ns, kh, kw) if sel is not None else (fo, f, kh, kw))
    _load().oracle_conv_accgrad(_p(x), _p(gy), _p(gw), S, f, fo, h, wd, kh, kw, sp, ns)
    return gw


def dft_r2c_1d(x, n):
    """x[B,n_in] -> complex128 [B,n/2+1]; x is zero-padded to n."""
    x = _d(x)
    B, n_in = x.shape
    assert n_in <= n
    out = np.empty((B, n // 2 + 1, 2))
    _load().oracle_dft_r2c_1d(_p(x), _p(out), B, n_in, n)
    return out[..., 0] + 1j * out[..., 1]


def idft_c2r_1d(X, n, n_out):
    """complex [B,n/2+1] -> real [B,n_out] (true inverse, scaled by 1/n, cropped)."""
    X = np.asarray(X)
    B = X.shape[0]
    assert X.shape[1] == n // 2 + 1 and n_out <= n
    buf = _d(np.stack([X.real, X.imag], axis=-1))
    out = np.empty((B, n_out))
    _load().oracle_idft_c2r_1d(_p(buf), _p(out), B, n, n_out)
    return out


def dft_r2c_2d(x, n):
    """x[B,h_in,w_in] -> complex128 [B,n,n/2+1]; x is zero-padded to n x n."""
    x = _d(x)
    B, h_in, w_in = x.shape
    assert h_in <= n and w_in <= n
    out = np.empty((B, n, n // 2 + 1, 2))
    _load().oracle_dft_r2c_2d(_p(x), _p(out), B, h_in, w_in, n)
    return out[..., 0] + 1j * out[..., 1]


def idft_c2r_2d(X, n, h_out, w_out):
    """complex [B,n,n/2+1] -> real [B,h_out,w_out] (scaled by 1/n^2, cropped at the origin)."""
    X = np.asarray(X)
    B = X.shape[0]
    assert X.shape[1:] == (n, n // 2 + 1) and h_out <= n and w_out <= n
    buf = _d(np.stack([X.real, X.imag], axis=-1))
    out = np.empty((B, h_out, w_out))
    _load().oracle_idft_c2r_2d(_p(buf), _p(out), B, n, h_out, w_out)
    return out


def dft2_bruteforce(x):
    """Full complex n x n DFT of one real n x n array by the four-index definition."""
    x = _d(x)
    n = x.shape[0]
    assert x.shape == (n, n)
    out = np.empty((n, n, 2))
    _load().oracle_dft2_bruteforce(_p(x), _p(out), n)
    return out[..., 0] + 1j * out[..., 1]
