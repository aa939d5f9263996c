"""Parity of the stand-alone FFT entry points against the naive-DFT oracle (GPU, via the C ABI).

Bound: max|err| / max|ref| <= 1e-5 (fp32 transforms of length <= 128 per dimension, 256 in
1-D, powers of two and sizes with one factor 3, 5 or 7: the error of an n-point fp32 FFT grows like log2(n) * 6e-8 relative to the largest output)."""
import numpy as np
import pytest

import oracle
from paper_1412_7580_amd import synth

pytestmark = pytest.mark.gpu
TOL = 1e-5
POW2 = [8, 16, 32, 64, 128]                            # the sizes of Section 5 of the paper
MIXED = [10, 12, 14, 18, 20, 24, 28, 36, 40, 48, 56, 80, 96, 112]   # 2^a * {3, 5, 7, 9}: bases of Section 3.2
SIZES = sorted(POW2 + MIXED)
SIZES_1D = SIZES + [160, 192, 224, 256]   # the 1-D calls go one octave further (Section 5.3)


@pytest.fixture(scope="module")
def hd(lib):
    h = lib.Handle(0)
    yield h
    h.close()


def _relerr(got, ref):
    return float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))


def _c(t):
    a = t.cpu().numpy().astype(np.float64)
    return a[..., 0] + 1j * a[..., 1]


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def _cdev(X):
    return _dev(np.stack([X.real, X.imag], axis=-1))


# batch sizes: one ragged block, several blocks with a ragged tail, a single signal
@pytest.mark.parametrize("n", SIZES_1D)
@pytest.mark.parametrize("B", [1, 2, 3, 700, 1025])
def test_r2c_1d(hd, n, B):
    x = synth.normal01(11, 0, (B, n - 3))
    got = _c(hd.fft_r2c_1d(_dev(x), n))
    assert _relerr(got, oracle.dft_r2c_1d(x, n)) <= TOL


@pytest.mark.parametrize("n", SIZES_1D)
def test_r2c_1d_every_input_length(hd, n):
    for n_in in sorted({1, 2, 3, n // 2, n // 2 + 1, n - 1, n}):
        x = synth.normal01(12, 1, (37, n_in))
        got = _c(hd.fft_r2c_1d(_dev(x), n))
        assert _relerr(got, oracle.dft_r2c_1d(x, n)) <= TOL, n_in


@pytest.mark.parametrize("n", SIZES_1D)
@pytest.mark.parametrize("B", [1, 5, 513])
def test_c2r_1d(hd, n, B):
    x = synth.normal01(13, 2, (B, n))
    X = oracle.dft_r2c_1d(x, n)
    Xf = X.astype(np.complex64).astype(np.complex128)   # what the device actually receives
    for n_out in sorted({1, 2, n - 3, n}):
        got = hd.fft_c2r_1d(_cdev(Xf), n, n_out).cpu().numpy().astype(np.float64)
        assert _relerr(got, oracle.idft_c2r_1d(Xf, n, n_out)) <= TOL, n_out


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("B", [1, 3, 70])
def test_r2c_2d(hd, n, B):
    x = synth.normal01(14, 3, (B, n - 3, n - 3))
    got = _c(hd.fft_r2c_2d(_dev(x), n))
    assert _relerr(got, oracle.dft_r2c_2d(x, n)) <= TOL


@pytest.mark.parametrize("n", SIZES)
def test_r2c_2d_shapes(hd, n):
    for (h_in, w_in) in [(1, 1), (n, n), (3, n - 1), (n, 2), (n // 2 + 1, n // 2), (2, 5)]:
        x = synth.normal01(15, 4, (5, h_in, w_in))
        got = _c(hd.fft_r2c_2d(_dev(x), n))
        assert _relerr(got, oracle.dft_r2c_2d(x, n)) <= TOL, (h_in, w_in)


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("B", [1, 3, 67])
def test_c2r_2d(hd, n, B):
    x = synth.normal01(16, 5, (B, n, n))
    X = oracle.dft_r2c_2d(x, n).astype(np.complex64).astype(np.complex128)
    for (h_out, w_out) in [(n, n), (n - 3, n - 3), (1, 1), (3, n - 1), (n, 2)]:
        got = hd.fft_c2r_2d(_cdev(X), n, h_out, w_out).cpu().numpy().astype(np.float64)
        assert _relerr(got, oracle.idft_c2r_2d(X, n, h_out, w_out)) <= TOL, (h_out, w_out)


def _random_real_signal_spectrum(seed, B, n):
    """A random complex half spectrum [B, n, n/2+1] that is the transform of SOME real n x n
    signal without being computed from one: columns 0 < k2 < n/2 are free; the two
    self-conjugate columns k2 = 0 and k2 = n/2 are made Hermitian along k1
    (X[k1] = conj(X[n - k1]), real at k1 = 0 and n/2), which is the precondition of the 2-D
    inverse."""
    X = synth.normal01(seed, 0, (B, n, n // 2 + 1)) + 1j * synth.normal01(seed, 1, (B, n, n // 2 + 1))
    for k2 in (0, n // 2):
        col = X[:, :, k2]
        col = 0.5 * (col + np.conj(col[:, (-np.arange(n)) % n]))
        X[:, :, k2] = col
    return X.astype(np.complex64).astype(np.complex128)


@pytest.mark.parametrize("n", [8, 12, 16, 28, 32, 64, 128])
def test_c2r_2d_symmetrised_random_spectrum(hd, n):
    """2-D inverse of spectra that no forward transform produced: random bins, with only the
    columns k2 = 0 and n/2 symmetrised along k1 as the header requires.  (Without that symmetry
    the result is unspecified: the kernel packs the two columns into one complex line on the
    assumption that their column-inverse is real, while the oracle drops the imaginary part.)"""
    B = 9
    X = _random_real_signal_spectrum(31, B, n)
    for (h_out, w_out) in [(n, n), (n - 3, n - 3), (5, n)]:
        got = hd.fft_c2r_2d(_cdev(X), n, h_out, w_out).cpu().numpy().astype(np.float64)
        assert _relerr(got, oracle.idft_c2r_2d(X, n, h_out, w_out)) <= TOL, (h_out, w_out)


@pytest.mark.parametrize("dim", [1, 2])
@pytest.mark.parametrize("n", POW2)
def test_sweep_roundtrip_subset(hd, dim, n):
    """The FFT-sweep workload at a reduced batch: R2C from size n-3 then C2R cropped back."""
    B = 4099
    x = synth.fft_sweep_input(dim, n, 0, B)
    if dim == 1:
        X = hd.fft_r2c_1d(_dev(x), n)
        back = hd.fft_c2r_1d(X, n, n - 3)
        ref = oracle.dft_r2c_1d(x[:64], n)
    else:
        B = 257 if n >= 64 else B
        x = x[:B]
        X = hd.fft_r2c_2d(_dev(x), n)
        back = hd.fft_c2r_2d(X, n, n - 3, n - 3)
        ref = oracle.dft_r2c_2d(x[:16], n)
    assert _relerr(_c(X)[: len(ref)], ref) <= TOL
    assert _relerr(back.cpu().numpy().astype(np.float64), x.astype(np.float64)) <= TOL


def test_argument_errors(hd, lib):
    import torch
    x = torch.zeros((4, 20), device="cuda")
    with pytest.raises(lib.FFTConvError, match="unsupported"):
        hd.fft_r2c_1d(x, 44)            # 2^2 * 11: no such size
    with pytest.raises(lib.FFTConvError, match="invalid"):
        hd.fft_r2c_1d(x, 16)            # n_in > n
    with pytest.raises(lib.FFTConvError, match="unsupported"):
        hd.fft_r2c_2d(torch.zeros((1, 4, 4), device="cuda"), 256)
    with pytest.raises(lib.FFTConvError, match="unsupported"):
        hd.fft_r2c_1d(torch.zeros((1, 4), device="cuda"), 512)
    # an empty batch is a no-op, not an error
    out = hd.fft_r2c_1d(torch.zeros((0, 5), device="cuda"), 8)
    assert out.shape == (0, 5, 2)


@pytest.mark.parametrize("dim", [1, 2])
@pytest.mark.parametrize("n", POW2)
def test_sweep_full_size(hd, dim, n):
    """The FFT-sweep workload at its full size (256 MiB of input, the launch configuration the
    benchmark times): R2C checked against the oracle on the first, the last and a seeded sample
    of transforms; the C2R round trip checked against the input over the whole batch."""
    import torch
    B = synth.fft_sweep_batch(dim, n)
    x = synth.fft_sweep_input(dim, n, 0, B)
    dx = _dev(x)
    rng = np.random.default_rng(n * 10 + dim)
    sel = np.unique(np.concatenate([[0, B - 1], rng.integers(0, B, 510 if dim == 1 else 62)]))
    if dim == 1:
        X = hd.fft_r2c_1d(dx, n)
        back = hd.fft_c2r_1d(X, n, n - 3)
        ref = oracle.dft_r2c_1d(x[sel], n)
    else:
        X = hd.fft_r2c_2d(dx, n)
        back = hd.fft_c2r_2d(X, n, n - 3, n - 3)
        ref = oracle.dft_r2c_2d(x[sel], n)
    got = _c(X[torch.from_numpy(sel).cuda()])
    assert _relerr(got, ref) <= TOL
    err = float((back - dx).abs().max()) / float(dx.abs().max())
    assert err <= TOL


@pytest.mark.parametrize("n", [2, 4])
def test_smallest_sizes(hd, n):
    """n = 2 and 4, the low end of the range of Section 5: every input length, ragged batches,
    both dimensions, forward against the oracle and the inverse against the input."""
    for B in (1, 3, 2051):
        for n_in in range(1, n + 1):
            x = synth.normal01(21, n, (B, n_in))
            X = hd.fft_r2c_1d(_dev(x), n)
            assert _relerr(_c(X), oracle.dft_r2c_1d(x, n)) <= TOL, (B, n_in)
            back = hd.fft_c2r_1d(X, n, n_in).cpu().numpy().astype(np.float64)
            assert np.max(np.abs(back - x)) <= TOL * max(1.0, np.max(np.abs(x))), (B, n_in)
    for B in (1, 5, 300):
        for (h_in, w_in) in [(1, 1), (n, n), (1, n), (n, 1), (n - 1, n)]:
            x = synth.normal01(22, n, (B, h_in, w_in))
            X = hd.fft_r2c_2d(_dev(x), n)
            assert _relerr(_c(X), oracle.dft_r2c_2d(x, n)) <= TOL, (B, h_in, w_in)
            back = hd.fft_c2r_2d(X, n, h_in, w_in).cpu().numpy().astype(np.float64)
            assert np.max(np.abs(back - x)) <= TOL * max(1.0, np.max(np.abs(x))), (B, h_in, w_in)
