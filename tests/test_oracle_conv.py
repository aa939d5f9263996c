"""Pins for the time-domain oracle (oracle_conv_*): each test would fail for a
plausible slip (dropped term, flipped kernel, swapped operands, wrong index)."""
import os

import numpy as np
import pytest
import scipy.signal

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rand(rng, *shape):
    return rng.uniform(-1, 1, size=shape)


def _read_hand():
    d = {}
    for line in open(os.path.join(GOLD, "hand_conv_3x3.txt")):
        if line.startswith("#") or not line.strip():
            continue
        t = line.split()
        d[t[0]] = np.array([float(v) for v in t[3:]]).reshape(int(t[1]), int(t[2]))
    return d


def test_hand_example():
    d = _read_hand()
    x, w, gy = d["x"][None, None], d["w"][None, None], d["gy"][None, None]
    assert np.array_equal(oracle.conv_fprop(x, w)[0, 0], d["y"])
    assert np.array_equal(oracle.conv_bprop(gy, w, 3, 3)[0, 0], d["gx"])
    assert np.array_equal(oracle.conv_accgrad(x, gy)[0, 0], d["gw"])


def _brute(x, w, gy):
    """Second, independent form: scalar loops over every index of the definitions."""
    S, f, h, wd = x.shape
    fo, _, kh, kw = w.shape
    oh, ow = h - kh + 1, wd - kw + 1
    y = np.zeros((S, fo, oh, ow)); gx = np.zeros_like(x); gw = np.zeros_like(w)
    for s in range(S):
        for j in range(fo):
            for i in range(f):
                for a in range(oh):
                    for b in range(ow):
                        for u in range(kh):
                            for v in range(kw):
                                y[s, j, a, b] += x[s, i, a + u, b + v] * w[j, i, u, v]
                                gx[s, i, a + u, b + v] += gy[s, j, a, b] * w[j, i, u, v]
                                gw[j, i, u, v] += gy[s, j, a, b] * x[s, i, a + u, b + v]
    return y, gx, gw


@pytest.mark.parametrize("S,f,fo,h,wd,kh,kw", [(2, 3, 2, 7, 6, 3, 2), (1, 1, 3, 5, 5, 5, 5), (3, 2, 1, 4, 7, 1, 3)])
def test_bruteforce_tiny(S, f, fo, h, wd, kh, kw):
    rng = np.random.default_rng(10)
    x, w, gy = _rand(rng, S, f, h, wd), _rand(rng, fo, f, kh, kw), _rand(rng, S, fo, h - kh + 1, wd - kw + 1)
    y, gx, gw = _brute(x, w, gy)
    np.testing.assert_allclose(oracle.conv_fprop(x, w), y, rtol=0, atol=1e-13)
    np.testing.assert_allclose(oracle.conv_bprop(gy, w, h, wd), gx, rtol=0, atol=1e-13)
    np.testing.assert_allclose(oracle.conv_accgrad(x, gy), gw, rtol=0, atol=1e-13)


def test_library_single_plane():
    """f = f' = S = 1 reduces to scipy's 2-D correlate / convolve."""
    rng = np.random.default_rng(11)
    x, w = _rand(rng, 9, 11), _rand(rng, 4, 3)
    gy = _rand(rng, 6, 9)
    np.testing.assert_allclose(oracle.conv_fprop(x[None, None], w[None, None])[0, 0],
                               scipy.signal.correlate2d(x, w, mode="valid"), atol=1e-13)
    np.testing.assert_allclose(oracle.conv_bprop(gy[None, None], w[None, None], 9, 11)[0, 0],
                               scipy.signal.convolve2d(gy, w, mode="full"), atol=1e-13)
    np.testing.assert_allclose(oracle.conv_accgrad(x[None, None], gy[None, None])[0, 0],
                               scipy.signal.correlate2d(x, gy, mode="valid"), atol=1e-13)


def test_impulses():
    rng = np.random.default_rng(12)
    h = wd = 6; kh = kw = 3
    w = _rand(rng, 1, 1, kh, kw)
    p, q = 3, 2
    x = np.zeros((1, 1, h, wd)); x[0, 0, p, q] = 1.0
    y = oracle.conv_fprop(x, w)[0, 0]
    for a in range(h - kh + 1):
        for b in range(wd - kw + 1):
            u, v = p - a, q - b
            exp = w[0, 0, u, v] if 0 <= u < kh and 0 <= v < kw else 0.0
            assert y[a, b] == exp
    # a delta kernel at (u0,v0) shifts the input
    x = _rand(rng, 1, 1, h, wd)
    wdl = np.zeros((1, 1, kh, kw)); wdl[0, 0, 2, 1] = 1.0
    assert np.array_equal(oracle.conv_fprop(x, wdl)[0, 0], x[0, 0, 2:2 + 4, 1:1 + 4])
    # bprop of a delta gy at (a0,b0) pastes the (unflipped) kernel at (a0,b0)
    gy = np.zeros((1, 1, 4, 4)); gy[0, 0, 1, 2] = 1.0
    gx = oracle.conv_bprop(gy, w, h, wd)[0, 0]
    exp = np.zeros((h, wd)); exp[1:1 + kh, 2:2 + kw] = w[0, 0]
    assert np.array_equal(gx, exp)


def test_1x1_kernel_is_matmul():
    rng = np.random.default_rng(13)
    S, f, fo, h, wd = 3, 5, 4, 4, 3
    x, w = _rand(rng, S, f, h, wd), _rand(rng, fo, f, 1, 1)
    gy = _rand(rng, S, fo, h, wd)
    np.testing.assert_allclose(oracle.conv_fprop(x, w), np.einsum("sihw,ji->sjhw", x, w[:, :, 0, 0]), atol=1e-13)
    np.testing.assert_allclose(oracle.conv_bprop(gy, w, h, wd), np.einsum("sjhw,ji->sihw", gy, w[:, :, 0, 0]), atol=1e-13)
    np.testing.assert_allclose(oracle.conv_accgrad(x, gy)[:, :, 0, 0], np.einsum("sjhw,sihw->ji", gy, x), atol=1e-13)


def test_adjoint_identity():
    """<fprop(x,w),gy> = <x,bprop(gy,w)> = <w,accGrad(x,gy)>: ties the three passes."""
    rng = np.random.default_rng(14)
    S, f, fo, h, wd, kh, kw = 3, 4, 5, 9, 8, 4, 3
    x, w, gy = _rand(rng, S, f, h, wd), _rand(rng, fo, f, kh, kw), _rand(rng, S, fo, h - kh + 1, wd - kw + 1)
    a = np.sum(oracle.conv_fprop(x, w) * gy)
    b = np.sum(x * oracle.conv_bprop(gy, w, h, wd))
    c = np.sum(w * oracle.conv_accgrad(x, gy))
    assert abs(a - b) < 1e-11 and abs(a - c) < 1e-11 and abs(a) > 1e-3
    d = _read_hand()
    assert np.sum(d["y"] * d["gy"]) == np.sum(d["x"] * d["gx"]) == np.sum(d["w"] * d["gw"]) == -16


def test_linearity_and_plane_sum():
    rng = np.random.default_rng(15)
    S, f, fo, h, wd, kh, kw = 2, 2, 2, 6, 6, 3, 3
    x1, x2, w = _rand(rng, S, f, h, wd), _rand(rng, S, f, h, wd), _rand(rng, fo, f, kh, kw)
    np.testing.assert_allclose(oracle.conv_fprop(2 * x1 - 3 * x2, w),
                               2 * oracle.conv_fprop(x1, w) - 3 * oracle.conv_fprop(x2, w), atol=1e-12)
    parts = sum(oracle.conv_fprop(x1[:, i:i + 1], w[:, i:i + 1]) for i in range(f))
    np.testing.assert_allclose(oracle.conv_fprop(x1, w), parts, atol=1e-13)


def test_finite_difference():
    rng = np.random.default_rng(16)
    S, f, fo, h, wd, kh, kw = 2, 2, 3, 5, 6, 2, 3
    x, w, gy = _rand(rng, S, f, h, wd), _rand(rng, fo, f, kh, kw), _rand(rng, S, fo, h - kh + 1, wd - kw + 1)
    L = lambda xx, ww: np.sum(oracle.conv_fprop(xx, ww) * gy)
    gx, gw = oracle.conv_bprop(gy, w, h, wd), oracle.conv_accgrad(x, gy)
    e = 1e-5
    for idx in [(0, 1, 2, 3), (1, 0, 4, 0)]:
        d = np.zeros_like(x); d[idx] = e
        assert abs((L(x + d, w) - L(x - d, w)) / (2 * e) - gx[idx]) < 1e-8
    for idx in [(2, 1, 1, 2), (0, 0, 0, 0)]:
        d = np.zeros_like(w); d[idx] = e
        assert abs((L(x, w + d) - L(x, w - d)) / (2 * e) - gw[idx]) < 1e-8


def test_plane_selection_matches_full():
    rng = np.random.default_rng(17)
    S, f, fo, h, wd, kh, kw = 3, 2, 4, 6, 5, 3, 2
    x, w, gy = _rand(rng, S, f, h, wd), _rand(rng, fo, f, kh, kw), _rand(rng, S, fo, h - kh + 1, wd - kw + 1)
    sel = [0, 5, 11, 7]
    assert np.array_equal(oracle.conv_fprop(x, w, sel), oracle.conv_fprop(x, w).reshape(S * fo, 4, 4)[sel])
    sel = [5, 0, 3]
    assert np.array_equal(oracle.conv_bprop(gy, w, h, wd, sel), oracle.conv_bprop(gy, w, h, wd).reshape(S * f, h, wd)[sel])
    sel = [7, 1]
    assert np.array_equal(oracle.conv_accgrad(x, gy, sel), oracle.conv_accgrad(x, gy).reshape(fo * f, kh, kw)[sel])
