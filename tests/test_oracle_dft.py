"""Pins for the naive-DFT oracle and for its agreement with the direct passes."""
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")
SIZES = [8, 10, 12, 14, 16, 18, 20, 28, 32, 36, 56, 64, 96, 128]   # powers of two and sizes with a factor 3, 5, 7 or 9


def test_closed_forms_from_fixture():
    for line in open(os.path.join(GOLD, "dft_closed_forms.txt")):
        if line.startswith("#") or not line.strip():
            continue
        head, xs, Xs = [p.split() for p in line.split("|")]
        n = int(head[1])
        x = np.array([float(v) for v in xs])
        v = np.array([float(t) for t in Xs]).reshape(-1, 2)
        X = oracle.dft_r2c_1d(x[None], n)[0]
        np.testing.assert_allclose(X, v[:, 0] + 1j * v[:, 1], atol=1e-14)


@pytest.mark.parametrize("n", SIZES)
def test_delta_constant_cosine(n):
    d = np.zeros((1, n)); d[0, 0] = 1
    np.testing.assert_allclose(oracle.dft_r2c_1d(d, n)[0], np.ones(n // 2 + 1), atol=1e-14)
    c = np.full((1, n), 2.5)
    e = np.zeros(n // 2 + 1, complex); e[0] = 2.5 * n
    np.testing.assert_allclose(oracle.dft_r2c_1d(c, n)[0], e, atol=1e-12)
    m = 3
    x = np.cos(2 * np.pi * m * np.arange(n) / n)[None]
    e = np.zeros(n // 2 + 1, complex); e[m] = n / 2
    np.testing.assert_allclose(oracle.dft_r2c_1d(x, n)[0], e, atol=1e-12)
    x = np.sin(2 * np.pi * m * np.arange(n) / n)[None]     # sign of the exponent
    e = np.zeros(n // 2 + 1, complex); e[m] = -1j * n / 2
    np.testing.assert_allclose(oracle.dft_r2c_1d(x, n)[0], e, atol=1e-12)


@pytest.mark.parametrize("n", SIZES)
def test_shift_parseval_inverse_1d(n):
    rng = np.random.default_rng(n)
    x = rng.standard_normal((4, n))
    X = oracle.dft_r2c_1d(x, n)
    k = np.arange(n // 2 + 1)
    Xs = oracle.dft_r2c_1d(np.roll(x, 3, axis=1), n)
    np.testing.assert_allclose(Xs, X * np.exp(-2j * np.pi * 3 * k / n), atol=1e-11)
    wgt = np.full(n // 2 + 1, 2.0); wgt[0] = wgt[-1] = 1.0
    np.testing.assert_allclose((x ** 2).sum(1), (wgt * np.abs(X) ** 2).sum(1) / n, rtol=1e-12)
    np.testing.assert_allclose(oracle.idft_c2r_1d(X, n, n), x, atol=1e-12)
    np.testing.assert_allclose(oracle.idft_c2r_1d(X, n, n - 3), x[:, :n - 3], atol=1e-12)
    # implicit zero-padding n-3 -> n equals the transform of the explicitly padded signal
    xp = x.copy(); xp[:, n - 3:] = 0
    np.testing.assert_allclose(oracle.dft_r2c_1d(x[:, :n - 3], n), oracle.dft_r2c_1d(xp, n), atol=1e-12)
    # library routine
    np.testing.assert_allclose(X, np.fft.rfft(x, axis=1), atol=1e-11)


def test_c2r_ignores_imag_of_self_conjugate_bins():
    n = 16
    rng = np.random.default_rng(3)
    X = oracle.dft_r2c_1d(rng.standard_normal((2, n)), n)
    Y = X.copy(); Y[:, 0] += 0.7j; Y[:, -1] -= 0.3j
    np.testing.assert_allclose(oracle.idft_c2r_1d(Y, n, n), oracle.idft_c2r_1d(X, n, n), atol=1e-14)


@pytest.mark.parametrize("n", [8, 12, 14, 16])
def test_2d_vs_bruteforce_and_hermitian(n):
    rng = np.random.default_rng(20 + n)
    x = rng.standard_normal((n, n))
    full = oracle.dft2_bruteforce(x)
    X = oracle.dft_r2c_2d(x[None], n)[0]
    np.testing.assert_allclose(X, full[:, :n // 2 + 1], atol=1e-11)
    k = np.arange(n)
    np.testing.assert_allclose(full, np.conj(full[np.ix_((-k) % n, (-k) % n)]), atol=1e-11)


@pytest.mark.parametrize("n", SIZES)
def test_2d_library_padding_inverse(n):
    rng = np.random.default_rng(30 + n)
    B = 2
    x = rng.standard_normal((B, n - 3, n - 3))
    xp = np.zeros((B, n, n)); xp[:, :n - 3, :n - 3] = x
    X = oracle.dft_r2c_2d(x, n)
    np.testing.assert_allclose(X, np.fft.rfft2(xp), atol=1e-10)
    np.testing.assert_allclose(oracle.idft_c2r_2d(X, n, n - 3, n - 3), x, atol=1e-12)
    np.testing.assert_allclose(oracle.idft_c2r_2d(X, n, n, n), xp, atol=1e-12)
    # rectangular crop and rectangular input
    xr = rng.standard_normal((B, 5, n - 1))
    Xr = oracle.dft_r2c_2d(xr, n)
    np.testing.assert_allclose(oracle.idft_c2r_2d(Xr, n, 5, n - 1), xr, atol=1e-12)
    np.testing.assert_allclose(oracle.idft_c2r_2d(Xr, n, 3, 2), xr[:, :3, :2], atol=1e-12)


def test_2d_axis_order():
    """A plane varying only along h must put its energy in column k2 = 0."""
    n = 8
    x = np.tile(np.cos(2 * np.pi * 2 * np.arange(n) / n)[:, None], (1, n))
    X = oracle.dft_r2c_2d(x[None], n)[0]
    e = np.zeros((n, n // 2 + 1), complex); e[2, 0] = e[6, 0] = n * n / 2
    np.testing.assert_allclose(X, e, atol=1e-11)


# the basis only has to hold the image: 13x13 on 14 and 27x25 on 28 (the bprop result then fills
# the basis up to its last row) as well as the powers of two
@pytest.mark.parametrize("h,wd,kh,kw,N", [(7, 7, 3, 3, 8), (13, 13, 3, 3, 16), (8, 6, 5, 2, 8), (16, 16, 9, 9, 16),
                                          (13, 13, 3, 3, 14), (27, 25, 5, 4, 28), (12, 12, 5, 5, 12)])
def test_convolution_theorem_all_passes(h, wd, kh, kw, N):
    """Section 2's frequency-domain identity, and the two 'similar' forms for
    bprop (no conjugate) and accGrad (conjugate on the gradient), checked
    between the two oracles before any GPU code exists."""
    rng = np.random.default_rng(40)
    S, f, fo = 2, 3, 2
    oh, ow = h - kh + 1, wd - kw + 1
    x = rng.uniform(-1, 1, (S, f, h, wd)); w = rng.uniform(-1, 1, (fo, f, kh, kw)); gy = rng.uniform(-1, 1, (S, fo, oh, ow))
    XF = oracle.dft_r2c_2d(x.reshape(-1, h, wd), N).reshape(S, f, N, N // 2 + 1)
    WF = oracle.dft_r2c_2d(w.reshape(-1, kh, kw), N).reshape(fo, f, N, N // 2 + 1)
    GF = oracle.dft_r2c_2d(gy.reshape(-1, oh, ow), N).reshape(S, fo, N, N // 2 + 1)
    YF = np.einsum("sipq,jipq->sjpq", XF, np.conj(WF))
    y = oracle.idft_c2r_2d(YF.reshape(-1, N, N // 2 + 1), N, oh, ow).reshape(S, fo, oh, ow)
    np.testing.assert_allclose(y, oracle.conv_fprop(x, w), atol=1e-11)
    GXF = np.einsum("sjpq,jipq->sipq", GF, WF)
    gx = oracle.idft_c2r_2d(GXF.reshape(-1, N, N // 2 + 1), N, h, wd).reshape(S, f, h, wd)
    np.testing.assert_allclose(gx, oracle.conv_bprop(gy, w, h, wd), atol=1e-11)
    GWF = np.einsum("sjpq,sipq->jipq", np.conj(GF), XF)
    gw = oracle.idft_c2r_2d(GWF.reshape(-1, N, N // 2 + 1), N, kh, kw).reshape(fo, f, kh, kw)
    np.testing.assert_allclose(gw, oracle.conv_accgrad(x, gy), atol=1e-11)
