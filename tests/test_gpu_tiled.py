"""Parity of the tiled passes (tiling of large inputs into small transforms, Section 6 of the
paper) against the time-domain oracle (GPU, C ABI).

Tiling changes how the result is computed, not what it is: the oracle is the same direct
definition as for the untiled passes and the bound is the same, max|err| / max|ref| <= 1e-4
over the whole output tensor."""
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


# (shape, tile basis): several tiles per image with ragged last tiles in one or both
# directions, rectangular images and kernels, a window larger than the image (one tile),
# plane counts that are not multiples of the kernels' plane tile, every basis up to 64, and
# the library's own choice (0).
TILED = [
    (dict(S=2, f=3, fo=4, h=20, w=20, kh=3, kw=3), 8),
    (dict(S=2, f=3, fo=2, h=21, w=17, kh=3, kw=5), 8),
    (dict(S=1, f=2, fo=3, h=40, w=33, kh=5, kw=5), 16),
    (dict(S=3, f=5, fo=3, h=37, w=41, kh=2, kw=4), 16),
    (dict(S=2, f=2, fo=2, h=30, w=30, kh=7, kw=7), 32),
    (dict(S=1, f=2, fo=2, h=70, w=50, kh=9, kw=3), 32),
    (dict(S=1, f=1, fo=2, h=100, w=90, kh=5, kw=5), 64),
    (dict(S=1, f=2, fo=1, h=90, w=130, kh=33, kw=17), 64),
    (dict(S=2, f=3, fo=3, h=45, w=45, kh=5, kw=5), 0),
    (dict(S=1, f=1, fo=1, h=9, w=9, kh=8, kw=8), 8),
    (dict(S=5, f=9, fo=7, h=24, w=24, kh=1, kw=1), 8),
    # widths, tile pitches and offsets that are multiples of 4: the 16-byte gather / scatter
    (dict(S=2, f=3, fo=2, h=40, w=40, kh=5, kw=5), 16),
    (dict(S=1, f=4, fo=3, h=64, w=48, kh=5, kw=5), 32),
    (dict(S=1, f=2, fo=2, h=37, w=44, kh=3, kw=9), 16),
    # one tile at the largest basis: the conv-layout kernels of basis 128
    (dict(S=1, f=2, fo=3, h=100, w=128, kh=9, kw=11), 128),
    # every basis with an odd factor (Section 3.2): several ragged tiles each, and plane counts
    # that do and do not fill the kernels' plane tiles
    (dict(S=2, f=3, fo=4, h=25, w=31, kh=3, kw=3), 12),
    (dict(S=2, f=5, fo=3, h=27, w=27, kh=3, kw=5), 14),
    (dict(S=1, f=4, fo=4, h=50, w=41, kh=5, kw=5), 20),
    (dict(S=3, f=2, fo=3, h=45, w=60, kh=7, kw=2), 24),
    (dict(S=2, f=3, fo=2, h=60, w=57, kh=5, kw=5), 28),
    (dict(S=1, f=2, fo=3, h=90, w=75, kh=9, kw=9), 40),
    (dict(S=1, f=3, fo=2, h=100, w=95, kh=11, kw=5), 48),
    (dict(S=1, f=2, fo=2, h=110, w=60, kh=7, kw=7), 56),
    (dict(S=1, f=2, fo=1, h=150, w=81, kh=5, kw=9), 80),
    (dict(S=1, f=1, fo=2, h=100, w=190, kh=13, kw=3), 96),
    (dict(S=1, f=2, fo=2, h=112, w=120, kh=9, kw=9), 112),
]
IDS = ["S{S}f{f}fo{fo}_{h}x{w}_k{kh}x{kw}".format(**c) + f"_n{n}" for c, n in TILED]


@pytest.mark.parametrize("cfg,tile_n", TILED, ids=IDS)
def test_tiled_passes(hd, cfg, tile_n):
    x, w, gy = synth.conv_inputs(seed=300, **cfg)
    dx, dw, dgy = _dev(x), _dev(w), _dev(gy)
    e = _relerr(_np(hd.fft_conv_fprop_tiled(dx, dw, tile_n)), oracle.conv_fprop(x, w))
    assert e <= TOL, ("fprop", e)
    e = _relerr(_np(hd.fft_conv_bprop_tiled(dgy, dw, cfg["h"], cfg["w"], tile_n)),
                oracle.conv_bprop(gy, w, cfg["h"], cfg["w"]))
    assert e <= TOL, ("bprop", e)
    e = _relerr(_np(hd.fft_conv_accgrad_tiled(dx, dgy, tile_n)), oracle.conv_accgrad(x, gy))
    assert e <= TOL, ("accgrad", e)


def test_tiled_equals_untiled_at_c2_shape(hd):
    """AlexNet-like second layer at a reduced plane count: tiled (basis 16) and untiled
    (basis 32) results agree with the oracle and hence with each other."""
    cfg = dict(S=8, f=16, fo=12, h=27, w=27, kh=5, kw=5)
    x, w, gy = synth.conv_inputs(seed=301, **cfg)
    dx, dw, dgy = _dev(x), _dev(w), _dev(gy)
    ref = oracle.conv_fprop(x, w)
    a, b = _np(hd.fft_conv_fprop_tiled(dx, dw, 16)), _np(hd.fft_conv_fprop(dx, dw))
    assert _relerr(a, ref) <= TOL and _relerr(b, ref) <= TOL
    ref = oracle.conv_accgrad(x, gy)
    a, b = _np(hd.fft_conv_accgrad_tiled(dx, dgy, 16)), _np(hd.fft_conv_accgrad(dx, dgy))
    assert _relerr(a, ref) <= TOL and _relerr(b, ref) <= TOL


def test_large_images_tile_by_themselves(hd):
    """Images beyond the largest basis (128): the ordinary entry points, and the
    transform-reuse pair, tile on their own."""
    import torch
    cfg = dict(S=1, f=2, fo=3, h=150, w=137, kh=5, kw=3)
    x, w, gy = synth.conv_inputs(seed=302, **cfg)
    dx, dw, dgy = _dev(x), _dev(w), _dev(gy)
    ry, rgx, rgw = oracle.conv_fprop(x, w), oracle.conv_bprop(gy, w, cfg["h"], cfg["w"]), oracle.conv_accgrad(x, gy)
    assert _relerr(_np(hd.fft_conv_fprop(dx, dw)), ry) <= TOL
    assert _relerr(_np(hd.fft_conv_bprop(dgy, dw, cfg["h"], cfg["w"])), rgx) <= TOL
    assert _relerr(_np(hd.fft_conv_accgrad(dx, dgy)), rgw) <= TOL
    dims = (cfg["S"], cfg["f"], cfg["fo"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
    saved = torch.empty(hd.saved_bytes(*dims) // 4, device="cuda", dtype=torch.float32)
    assert saved.numel() > 0
    y = hd.fft_conv_fprop_save(dx, dw, saved)
    gx, gw = hd.fft_conv_backward(dgy, saved, cfg["f"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
    assert _relerr(_np(y), ry) <= TOL
    assert _relerr(_np(gx), rgx) <= TOL
    assert _relerr(_np(gw), rgw) <= TOL


def test_tiled_accgrad_scale_and_accumulate(hd):
    import torch
    cfg = dict(S=2, f=3, fo=2, h=26, w=22, kh=3, kw=3)
    x, w, gy = synth.conv_inputs(seed=303, **cfg)
    dx, dgy = _dev(x), _dev(gy)
    ref = oracle.conv_accgrad(x, gy)
    gw0 = torch.full((cfg["fo"], cfg["f"], cfg["kh"], cfg["kw"]), 2.0, device="cuda")
    got = hd.fft_conv_accgrad_tiled(dx, dgy, 8, gw=gw0, scale=0.5, accumulate=True)
    assert _relerr(_np(got), 2.0 + 0.5 * ref) <= TOL


def test_tiled_workspace_and_errors(hd, lib):
    import torch
    cfg = dict(S=2, f=2, fo=2, h=20, w=20, kh=3, kw=3)
    x, w, _ = synth.conv_inputs(seed=304, **cfg)
    dx, dw = _dev(x), _dev(w)
    dims = (cfg["S"], cfg["f"], cfg["fo"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
    need = hd.tiled_workspace_bytes(lib.FPROP, *dims, 8)
    assert need > 0
    ws = torch.empty(need // 4, device="cuda", dtype=torch.float32)
    y = hd.fft_conv_fprop_tiled(dx, dw, 8, ws=ws)
    assert _relerr(_np(y), oracle.conv_fprop(x, w)) <= TOL
    with pytest.raises(lib.FFTConvError, match="workspace too small"):
        hd.fft_conv_fprop_tiled(dx, dw, 8, ws=ws[: need // 4 - 64])
    for bad in (-1, 22, 256):
        with pytest.raises(lib.FFTConvError, match="invalid argument"):
            hd.fft_conv_fprop_tiled(dx, dw, bad)
    big_k = torch.zeros((1, 1, 9, 9), device="cuda")
    with pytest.raises(lib.FFTConvError, match="invalid argument"):      # basis smaller than the kernel
        hd.fft_conv_fprop_tiled(torch.zeros((1, 1, 20, 20), device="cuda"), big_k, 8)
    assert hd.tile_basis(20, 20, 3, 3, 16) == 16
    assert hd.tile_basis(200, 200, 5, 5, 0) in (8, 10, 12, 14, 16, 18, 20, 24, 28, 32, 36, 40, 48, 56, 64, 80, 96, 112, 128)
    assert hd.tile_basis(20, 20, 3, 3, 12) == 12
    assert hd.tile_basis(20, 20, 3, 3, 18) == 18
    assert hd.tile_basis(20, 20, 3, 3, 22) == 0


def test_tiled_is_deterministic(hd):
    cfg = dict(S=2, f=4, fo=4, h=30, w=30, kh=3, kw=3)
    x, w, gy = synth.conv_inputs(seed=305, **cfg)
    dx, dw, dgy = _dev(x), _dev(w), _dev(gy)
    a = hd.fft_conv_bprop_tiled(dgy, dw, cfg["h"], cfg["w"], 16).clone()
    b = hd.fft_conv_bprop_tiled(dgy, dw, cfg["h"], cfg["w"], 16)
    assert bool((a == b).all())


BASES = (8, 10, 12, 14, 16, 18, 20, 24, 28, 32, 36, 40, 48, 56, 64, 80, 96, 112, 128)


@pytest.mark.parametrize("n", [28, 32, 40, 56])
def test_named_basis_that_holds_the_image(hd, n):
    """tile_n >= max(h, w): the untiled pipeline at that basis (three frequency tensors, one
    transform per plane), for all three passes."""
    cfg = dict(S=3, f=5, fo=4, h=27, w=25, kh=5, kw=4)
    x, w, gy = synth.conv_inputs(seed=310, **cfg)
    dx, dw, dgy = _dev(x), _dev(w), _dev(gy)
    assert _relerr(_np(hd.fft_conv_fprop_tiled(dx, dw, n)), oracle.conv_fprop(x, w)) <= TOL
    assert _relerr(_np(hd.fft_conv_bprop_tiled(dgy, dw, 27, 25, n)), oracle.conv_bprop(gy, w, 27, 25)) <= TOL
    assert _relerr(_np(hd.fft_conv_accgrad_tiled(dx, dgy, n)), oracle.conv_accgrad(x, gy)) <= TOL
    T = {28: 16, 32: 8, 40: 4, 56: 4}[n]     # planes per tile of the layout
    bins = {28: 424, 32: 544, 40: 864, 56: 1632}[n]     # n * (n/2 + 1), padded to the layout's unit
    pad = lambda planes: -(-planes // T) * T
    assert hd.tiled_workspace_bytes(0, 3, 5, 4, 27, 25, 5, 4, n) == (pad(15) + pad(20) + pad(12)) * bins * 2 * 4


@pytest.mark.parametrize("n", [10, 18, 36])
def test_bases_with_a_factor_nine_or_ten(hd, n):
    """The sizes 10 = 2 x 5, 18 = 2 x 9 and 36 = 4 x 9: the ordinary calls take them for images
    that fit, and the three passes agree with the oracle, whole and as a tile basis."""
    cfg = dict(S=5, f=6, fo=9, h=n, w=n - 1, kh=3, kw=2)
    assert hd.layer_basis(n, n, 3, 3) == (n, n, False)
    x, w, gy = synth.conv_inputs(seed=330 + n, **cfg)
    dx, dw, dgy = _dev(x), _dev(w), _dev(gy)
    ref = (oracle.conv_fprop(x, w), oracle.conv_bprop(gy, w, cfg["h"], cfg["w"]), oracle.conv_accgrad(x, gy))
    got = (hd.fft_conv_fprop_tiled(dx, dw, n), hd.fft_conv_bprop_tiled(dgy, dw, cfg["h"], cfg["w"], n),
           hd.fft_conv_accgrad_tiled(dx, dgy, n))
    for g, r in zip(got, ref):
        assert _relerr(_np(g), r) <= TOL
    # a larger image cut into tiles of this basis
    big = dict(S=2, f=3, fo=4, h=3 * n + 1, w=2 * n + 5, kh=3, kw=3)
    x, w, gy = synth.conv_inputs(seed=340 + n, **big)
    dx, dw, dgy = _dev(x), _dev(w), _dev(gy)
    assert hd.tile_basis(big["h"], big["w"], 3, 3, n) == n
    ref = (oracle.conv_fprop(x, w), oracle.conv_bprop(gy, w, big["h"], big["w"]), oracle.conv_accgrad(x, gy))
    got = (hd.fft_conv_fprop_tiled(dx, dw, n), hd.fft_conv_bprop_tiled(dgy, dw, big["h"], big["w"], n),
           hd.fft_conv_accgrad_tiled(dx, dgy, n))
    for g, r in zip(got, ref):
        assert _relerr(_np(g), r) <= TOL


@pytest.mark.parametrize("n", [10, 12, 14, 16, 18, 20, 24, 28, 32])
@pytest.mark.parametrize("tiled", [False, True])
def test_backward_with_shared_launches(hd, n, tiled):
    """fft_conv_backward on the bases where both contractions and both inverse transforms share
    a launch (three launches in all): whole images and windows, with scale and accumulate on
    the weight gradients."""
    import torch
    h, w = (n - 1, n - 3) if not tiled else (2 * n + 3, n + 9)
    cfg = dict(S=4, f=8, fo=12, h=h, w=w, kh=3, kw=4)
    x, wt, gy = synth.conv_inputs(seed=350 + n, **cfg)
    dx, dw, dgy = _dev(x), _dev(wt), _dev(gy)
    dims = (cfg["S"], cfg["f"], cfg["fo"], h, w, cfg["kh"], cfg["kw"])
    saved = torch.empty(hd.saved_bytes_tiled(*dims, n) // 4, device="cuda")
    hd.fft_conv_fprop_save_tiled(dx, dw, n, saved)
    gw = torch.full((12, 8, 3, 4), 0.25, device="cuda")
    hd.set_profiling(True)
    gx, _ = hd.fft_conv_backward_tiled(dgy, saved, cfg["f"], h, w, cfg["kh"], cfg["kw"], n, gw=gw, scale=-0.5,
                                       accumulate=True)
    launches = len(hd.last_kernel_ms())
    hd.set_profiling(False)
    assert launches == 3
    assert _relerr(_np(gx), oracle.conv_bprop(gy, wt, h, w)) <= TOL
    assert _relerr(_np(gw), 0.25 - 0.5 * oracle.conv_accgrad(x, gy)) <= TOL
    # the same through separate passes
    gx2 = hd.fft_conv_bprop_tiled(dgy, dw, h, w, n)
    assert float((gx - gx2).abs().max()) <= 2e-5 * float(gx2.abs().max())


def test_autotune_basis(hd):
    """The measured choice is one of the candidate bases, and the outputs left behind are the
    chosen basis's results (checked against the oracle and against the tiled calls)."""
    import torch
    cfg = dict(S=4, f=8, fo=8, h=30, w=26, kh=3, kw=5)
    x, w, gy = synth.conv_inputs(seed=311, **cfg)
    dx, dw, dgy = _dev(x), _dev(w), _dev(gy)
    y, gx, gw = torch.empty_like(dgy), torch.empty_like(dx), torch.empty_like(dw)
    n, ms = hd.autotune_basis(dx, dw, dgy, y=y, gx=gx, gw=gw, reps=2)
    assert n in BASES and n >= 5 and ms > 0
    assert _relerr(_np(y), oracle.conv_fprop(x, w)) <= TOL
    assert _relerr(_np(gx), oracle.conv_bprop(gy, w, 30, 26)) <= TOL
    assert _relerr(_np(gw), oracle.conv_accgrad(x, gy)) <= TOL
    assert torch.equal(y, hd.fft_conv_fprop_tiled(dx, dw, n))
    assert torch.equal(gx, hd.fft_conv_bprop_tiled(dgy, dw, 30, 26, n))
    assert torch.equal(gw, hd.fft_conv_accgrad_tiled(dx, dgy, n))


@pytest.mark.parametrize("cfg,n", [(dict(S=3, f=4, fo=5, h=27, w=27, kh=5, kw=5), 32),     # named basis, untiled
                                   (dict(S=3, f=4, fo=5, h=27, w=27, kh=5, kw=5), 28),
                                   (dict(S=2, f=3, fo=4, h=45, w=50, kh=3, kw=5), 24)])    # tiled
def test_reuse_pair_on_a_named_basis(hd, cfg, n):
    """fft_conv_fprop_save_tiled + fft_conv_backward_tiled equal the three tiled passes."""
    import torch
    x, w, gy = synth.conv_inputs(seed=312, **cfg)
    dx, dw, dgy = _dev(x), _dev(w), _dev(gy)
    dims = (cfg["S"], cfg["f"], cfg["fo"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
    saved = torch.empty(hd.saved_bytes_tiled(*dims, n) // 4, device="cuda")
    assert saved.numel() > 0 and hd.backward_workspace_bytes_tiled(*dims, n) > 0
    y = hd.fft_conv_fprop_save_tiled(dx, dw, n, saved)
    gx, gw = hd.fft_conv_backward_tiled(dgy, saved, cfg["f"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"], n)
    assert _relerr(_np(y), oracle.conv_fprop(x, w)) <= TOL
    assert _relerr(_np(gx), oracle.conv_bprop(gy, w, cfg["h"], cfg["w"])) <= TOL
    assert _relerr(_np(gw), oracle.conv_accgrad(x, gy)) <= TOL
    assert torch.equal(y, hd.fft_conv_fprop_tiled(dx, dw, n))
    with pytest.raises(Exception, match="workspace too small"):
        hd.fft_conv_fprop_save_tiled(dx, dw, n, saved[:-64])
