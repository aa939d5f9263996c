"""Parity of the zero-padded passes (p_h, p_w of Section 2 of the paper) against the
time-domain oracle (GPU, C ABI).

The oracle has no notion of padding: the expected values are its results on explicitly padded
copies of x (fprop, accGrad), and the interior of its bprop result for the padded shape.
Bound as for the other passes: max|err| / max|ref| <= 1e-4 over the whole tensor."""
import numpy as np
import pytest

import oracle
from paper_1412_7580_amd import synth

pytestmark = pytest.mark.gpu
TOL = 1e-4


@pytest.fixture(scope="module")
def hd(lib):
    h = lib.Handle(0)
    yield h
    h.close()


def _relerr(got, ref):
    return float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def _np(t):
    return t.cpu().numpy().astype(np.float64)


# "same" convolutions (pad = (k-1)/2), asymmetric padding, padding larger than the kernel
# reach (all-zero border outputs), padded images that need one window, several windows, and
# more than the largest basis; plane counts that are not multiples of the kernels' tiles.
PADDED = [
    (dict(S=2, f=3, fo=4, h=13, w=13, kh=3, kw=3), 1, 1),
    (dict(S=3, f=2, fo=2, h=12, w=9, kh=5, kw=3), 2, 0),
    (dict(S=1, f=2, fo=3, h=10, w=11, kh=2, kw=4), 3, 5),
    (dict(S=2, f=4, fo=4, h=27, w=27, kh=5, kw=5), 2, 2),
    (dict(S=1, f=2, fo=2, h=60, w=60, kh=7, kw=7), 3, 3),
    (dict(S=1, f=1, fo=2, h=126, w=100, kh=3, kw=3), 2, 1),
    (dict(S=1, f=2, fo=1, h=140, w=131, kh=5, kw=5), 2, 2),
    (dict(S=4, f=8, fo=8, h=28, w=28, kh=5, kw=5), 2, 2),
]
IDS = ["S{S}f{f}fo{fo}_{h}x{w}_k{kh}x{kw}".format(**c) + f"_p{a}x{b}" for c, a, b in PADDED]


@pytest.mark.parametrize("cfg,ph,pw", PADDED, ids=IDS)
def test_padded_passes(hd, cfg, ph, pw):
    h, w = cfg["h"], cfg["w"]
    big = dict(cfg, h=h + 2 * ph, w=w + 2 * pw)
    xp, wt, gy = synth.conv_inputs(seed=400, **big)           # gy has the padded layer's output shape
    x = np.ascontiguousarray(xp[:, :, ph:ph + h, pw:pw + w])
    xpad = np.zeros_like(xp)
    xpad[:, :, ph:ph + h, pw:pw + w] = x
    dx, dw, dgy = _dev(x), _dev(wt), _dev(gy)
    e = _relerr(_np(hd.fft_conv_fprop_padded(dx, dw, ph, pw)), oracle.conv_fprop(xpad, wt))
    assert e <= TOL, ("fprop", e)
    ref = oracle.conv_bprop(gy, wt, h + 2 * ph, w + 2 * pw)[:, :, ph:ph + h, pw:pw + w]
    e = _relerr(_np(hd.fft_conv_bprop_padded(dgy, dw, h, w, ph, pw)), ref)
    assert e <= TOL, ("bprop", e)
    e = _relerr(_np(hd.fft_conv_accgrad_padded(dx, dgy, ph, pw)), oracle.conv_accgrad(xpad, gy))
    assert e <= TOL, ("accgrad", e)


@pytest.mark.parametrize("cfg,ph,pw", [PADDED[0], PADDED[3], PADDED[6], PADDED[7]],
                         ids=[IDS[0], IDS[3], IDS[6], IDS[7]])
def test_padded_reuse_pair(hd, cfg, ph, pw):
    """fprop_save + backward of a padded layer give, bit for bit, what the three padded passes
    give (which the test above checks against the oracle)."""
    import torch
    h, w = cfg["h"], cfg["w"]
    big = dict(cfg, h=h + 2 * ph, w=w + 2 * pw)
    xp, wt, gy = synth.conv_inputs(seed=402, **big)
    x = np.ascontiguousarray(xp[:, :, ph:ph + h, pw:pw + w])
    dx, dw, dgy = _dev(x), _dev(wt), _dev(gy)
    dims = (cfg["S"], cfg["f"], cfg["fo"], h, w, cfg["kh"], cfg["kw"])
    saved = torch.empty(hd.saved_bytes_padded(*dims, ph, pw) // 4, device="cuda", dtype=torch.float32)
    assert saved.numel() > 0 and hd.backward_workspace_bytes_padded(*dims, ph, pw) > 0
    y = hd.fft_conv_fprop_save_padded(dx, dw, ph, pw, saved)
    gx, gw = hd.fft_conv_backward_padded(dgy, saved, cfg["f"], h, w, cfg["kh"], cfg["kw"], ph, pw)
    assert torch.equal(y, hd.fft_conv_fprop_padded(dx, dw, ph, pw))
    assert torch.equal(gx, hd.fft_conv_bprop_padded(dgy, dw, h, w, ph, pw))
    assert torch.equal(gw, hd.fft_conv_accgrad_padded(dx, dgy, ph, pw))


def test_zero_padding_is_the_ordinary_pass(hd):
    cfg = dict(S=2, f=3, fo=2, h=14, w=14, kh=3, kw=3)
    x, wt, gy = synth.conv_inputs(seed=401, **cfg)
    dx, dw = _dev(x), _dev(wt)
    ref = oracle.conv_fprop(x, wt)
    assert _relerr(_np(hd.fft_conv_fprop_padded(dx, dw, 0, 0)), ref) <= TOL
    assert _relerr(_np(hd.fft_conv_fprop(dx, dw)), ref) <= TOL


def test_padded_errors_and_workspace(hd, lib):
    import torch
    x = torch.zeros((1, 1, 6, 6), device="cuda")
    k = torch.zeros((1, 1, 3, 3), device="cuda")
    with pytest.raises(lib.FFTConvError, match="invalid argument"):
        hd.fft_conv_fprop_padded(x, k, -1, 0, y=torch.zeros((1, 1, 2, 4), device="cuda"))
    with pytest.raises(lib.FFTConvError, match="invalid argument"):      # kernel larger than the padded image
        hd.fft_conv_fprop_padded(torch.zeros((1, 1, 2, 2), device="cuda"), torch.zeros((1, 1, 5, 5), device="cuda"),
                                 1, 1, y=torch.zeros((1, 1, 1, 1), device="cuda"))
    need = hd.padded_workspace_bytes(lib.FPROP, 1, 1, 1, 6, 6, 3, 3, 1, 1)
    assert need > 0
    ws = torch.empty(need // 4, device="cuda", dtype=torch.float32)
    hd.fft_conv_fprop_padded(x, k, 1, 1, ws=ws)
    with pytest.raises(lib.FFTConvError, match="workspace too small"):
        hd.fft_conv_fprop_padded(x, k, 1, 1, ws=ws[: need // 8])


@pytest.mark.parametrize("cfg,pad", [(dict(S=5, f=6, fo=7, h=13, w=13, kh=3, kw=3), (0, 0)),       # basis 14
                                     (dict(S=3, f=4, fo=5, h=27, w=25, kh=5, kw=5), (2, 2)),       # padded: windows
                                     (dict(S=2, f=3, fo=2, h=150, w=140, kh=7, kw=5), (0, 0)),     # tiled by itself
                                     (dict(S=2, f=8, fo=8, h=64, w=64, kh=31, kw=31), (0, 0))])    # basis 64
def test_weights_transformed_ahead(hd, lib, cfg, pad):
    """fft_conv_transform_weights once, then fprop and bprop for two different minibatches: equal
    to the ordinary (padded) passes bit for bit (same kernels on the same transforms) and to the
    oracle within the bound."""
    import torch
    ph, pw = pad
    h, w, kh, kw = cfg["h"], cfg["w"], cfg["kh"], cfg["kw"]
    big = dict(cfg, h=h + 2 * ph, w=w + 2 * pw)
    wf = None
    for S in (cfg["S"], 1):
        xp, wt, gy = synth.conv_inputs(seed=700 + S, **dict(big, S=S))
        x = np.ascontiguousarray(xp[:, :, ph:ph + h, pw:pw + w])
        xpad = np.zeros_like(xp)
        xpad[:, :, ph:ph + h, pw:pw + w] = x
        if wf is None:
            w0 = wt                                           # the weights of the first draw serve both minibatches
            wf = hd.fft_conv_transform_weights(_dev(w0), h, w, ph, pw)
            assert wf.numel() * 4 == hd.weights_bytes(cfg["f"], cfg["fo"], h, w, kh, kw, ph, pw) > 0
        dx, dw, dgy = _dev(x), _dev(w0), _dev(gy)
        y = hd.fft_conv_fprop_weights(dx, wf, cfg["fo"], kh, kw, ph, pw)
        gx = hd.fft_conv_bprop_weights(dgy, wf, cfg["f"], h, w, kh, kw, ph, pw)
        assert torch.equal(y, hd.fft_conv_fprop_padded(dx, dw, ph, pw))
        assert torch.equal(gx, hd.fft_conv_bprop_padded(dgy, dw, h, w, ph, pw))
        assert _relerr(_np(y), oracle.conv_fprop(xpad, w0)) <= TOL
        ref = oracle.conv_bprop(gy, w0, h + 2 * ph, w + 2 * pw)[:, :, ph:ph + h, pw:pw + w]
        assert _relerr(_np(gx), ref) <= TOL
    with pytest.raises(lib.FFTConvError, match="workspace too small"):
        hd.fft_conv_fprop_weights(dx, wf[:-64], cfg["fo"], kh, kw, ph, pw)
