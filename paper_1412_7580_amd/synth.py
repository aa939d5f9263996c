"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds none of the method's arithmetic: it only produces the fp32
arrays (uniform[-1,1] activations / weights / output gradients, N(0,1) signals)
that both the HIP path and the CPU oracle are fed.  The generator is
counter-based (splitmix64 finaliser applied to ``seed*2^40 + stream*2^36 +
index``), so any slice of a tensor can be generated without the rest, which is
what sampled parity checks at full benchmark sizes need.
"""
from __future__ import annotations

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z + np.uint64(0x9E3779B97F4A7C15)) & _M64
    z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
    z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
    return z ^ (z >> np.uint64(31))


def _bits(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    base = (int(seed) << 40) + (int(stream) << 36) + int(start)
    with np.errstate(over="ignore"):
        idx = np.arange(count, dtype=np.uint64) + np.uint64(base & 0xFFFFFFFFFFFFFFFF)
        return _mix(idx)


def uniform_pm1(seed: int, stream: int, shape, start: int = 0) -> np.ndarray:
    """fp32 i.i.d. uniform on [-1, 1): 24 random bits -> k/2^23 - 1."""
    count = int(np.prod(shape))
    b = _bits(seed, stream, start, count) >> np.uint64(40)
    return (b.astype(np.float32) * np.float32(2.0 ** -23) - np.float32(1.0)).reshape(shape)


def normal01(seed: int, stream: int, shape, start: int = 0) -> np.ndarray:
    """fp32 N(0,1) by Box-Muller on two counter-based uniforms per sample."""
    count = int(np.prod(shape))
    b = _bits(seed, stream, 2 * start, 2 * count) >> np.uint64(11)
    u1 = b[0::2].astype(np.float64)
    u2 = b[1::2].astype(np.float64)
    u1 = (u1 + 1.0) * 2.0 ** -53
    u2 = u2 * 2.0 ** -53
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return z.astype(np.float32).reshape(shape)


# The four convolution workloads (S, f, f', h, w, kh, kw, FFT size) and the
# FFT sweep named by the benchmark definition.  Index = configuration number.
CONV_CONFIGS = {
    "C1": dict(S=16, f=16, fo=16, h=13, w=13, kh=3, kw=3, N=16, passes=("fprop",)),
    "C2": dict(S=128, f=64, fo=64, h=27, w=27, kh=5, kw=5, N=32, passes=("fprop", "bprop", "accgrad")),
    "C3": dict(S=128, f=384, fo=384, h=13, w=13, kh=3, kw=3, N=16, passes=("fprop", "bprop", "accgrad")),
    "C4": dict(S=32, f=128, fo=128, h=64, w=64, kh=31, kw=31, N=64, passes=("fprop", "bprop", "accgrad")),
}
CONV_SEEDS = {"C1": 0, "C2": 1, "C3": 2, "C4": 3}
FFT_SWEEP_SEED = 4
FFT_SWEEP_SIZES = (8, 16, 32, 64, 128)


def conv_inputs(S, f, fo, h, w, kh, kw, seed, **_):
    """(x, w, gy) fp32, each i.i.d. uniform[-1,1], independent streams 0, 1, 2."""
    x = uniform_pm1(seed, 0, (S, f, h, w))
    wt = uniform_pm1(seed, 1, (fo, f, kh, kw))
    gy = uniform_pm1(seed, 2, (S, fo, h - kh + 1, w - kw + 1))
    return x, wt, gy


def fft_sweep_batch(dim: int, n: int, in_bytes: int = 1 << 28) -> int:
    """Batch count of the FFT sweep: as many (n-3)^dim fp32 signals as fit in_bytes."""
    return in_bytes // (4 * (n - 3) ** dim)


def fft_sweep_input(dim: int, n: int, first: int, count: int) -> np.ndarray:
    """Signals first..first+count-1 of the sweep input for (dim, n): N(0,1), size (n-3)^dim."""
    per = (n - 3) ** dim
    shape = (count, n - 3) if dim == 1 else (count, n - 3, n - 3)
    stream = (dim - 1) * 5 + FFT_SWEEP_SIZES.index(n)
    return normal01(FFT_SWEEP_SEED, stream, shape, start=first * per)
