"""Parity of fft_conv_fprop / bprop / accgrad against the time-domain oracle (GPU, C ABI).

Bound: max|err| / max|ref| <= 1e-4 over the whole output tensor."""
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


def _run_all(hd, cfg, seed, passes=("fprop", "bprop", "accgrad"), basis=None):
    """basis=None: the ordinary entry points (the library's own basis); a number: that Fourier
    basis through the *_tiled entry points (untiled pipeline when it holds the image)."""
    x, w, gy = synth.conv_inputs(seed=seed, **cfg)
    dx, dw, dgy = _dev(x), _dev(w), _dev(gy)
    errs = {}
    if "fprop" in passes:
        got = hd.fft_conv_fprop(dx, dw) if basis is None else hd.fft_conv_fprop_tiled(dx, dw, basis)
        errs["fprop"] = _relerr(_np(got), oracle.conv_fprop(x, w))
    if "bprop" in passes:
        got = (hd.fft_conv_bprop(dgy, dw, cfg["h"], cfg["w"]) if basis is None
               else hd.fft_conv_bprop_tiled(dgy, dw, cfg["h"], cfg["w"], basis))
        errs["bprop"] = _relerr(_np(got), oracle.conv_bprop(gy, w, cfg["h"], cfg["w"]))
    if "accgrad" in passes:
        got = hd.fft_conv_accgrad(dx, dgy) if basis is None else hd.fft_conv_accgrad_tiled(dx, dgy, basis)
        errs["accgrad"] = _relerr(_np(got), oracle.conv_accgrad(x, gy))
    return errs


# Small shapes spanning every basis size, ragged plane counts (not multiples of the plane
# tile or of the MFMA tile), rectangular inputs/kernels, kernel == input, 1x1 kernels.
SMALL = [
    dict(S=1, f=1, fo=1, h=5, w=5, kh=3, kw=3),
    dict(S=2, f=3, fo=5, h=8, w=8, kh=3, kw=3),
    dict(S=3, f=2, fo=4, h=7, w=6, kh=2, kw=4),
    dict(S=5, f=7, fo=3, h=13, w=13, kh=3, kw=3),
    dict(S=2, f=33, fo=35, h=16, w=16, kh=5, kw=5),
    dict(S=34, f=5, fo=6, h=12, w=9, kh=12, kw=9),
    dict(S=4, f=6, fo=5, h=27, w=27, kh=5, kw=5),
    dict(S=3, f=5, fo=2, h=32, w=20, kh=1, kw=1),
    dict(S=2, f=3, fo=4, h=33, w=40, kh=7, kw=3),
    dict(S=3, f=2, fo=3, h=64, w=64, kh=31, kw=31),
    dict(S=2, f=2, fo=2, h=100, w=128, kh=9, kw=11),
    dict(S=70, f=40, fo=72, h=9, w=9, kh=3, kw=3),
    # fprop contraction of 144 bins x (4 x 2) tiles = 1152 workgroups: a short last round, whose
    # tiles are cut into quadrants (ragged ones, and quadrants wholly outside the matrix)
    dict(S=200, f=20, fo=72, h=13, w=13, kh=3, kw=3),
]


@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: "S{S}f{f}fo{fo}_{h}x{w}_k{kh}x{kw}".format(**c))
def test_small_shapes(hd, cfg):
    errs = _run_all(hd, cfg, seed=100)
    for k, e in errs.items():
        assert e <= TOL, (k, e)


# The benchmark configurations name their Fourier basis (16, 32, 16); the library by itself
# takes the smallest basis that holds the image (14, 28, 14).  Both are checked at full size.
@pytest.mark.parametrize("named", [False, True], ids=["library_basis", "named_basis"])
def test_config_c1_fprop(hd, named):
    cfg = synth.CONV_CONFIGS["C1"]
    errs = _run_all(hd, cfg, seed=synth.CONV_SEEDS["C1"], passes=cfg["passes"], basis=cfg["N"] if named else None)
    assert errs["fprop"] <= TOL


@pytest.mark.parametrize("named", [False, True], ids=["library_basis", "named_basis"])
@pytest.mark.parametrize("name", ["C2", "C3"])
def test_config_full_tensor(hd, name, named):
    cfg = synth.CONV_CONFIGS[name]
    errs = _run_all(hd, cfg, seed=synth.CONV_SEEDS[name], basis=cfg["N"] if named else None)
    for k, e in errs.items():
        assert e <= TOL, (name, k, e)


def test_config_c4_sampled_planes(hd):
    """Large-kernel layer at full size; the oracle evaluates a seeded sample of output planes
    (all pixels of each), the GPU computes everything in the benchmark's launch configuration."""
    cfg = synth.CONV_CONFIGS["C4"]
    seed = synth.CONV_SEEDS["C4"]
    x, w, gy = synth.conv_inputs(seed=seed, **cfg)
    dx, dw, dgy = _dev(x), _dev(w), _dev(gy)
    S, f, fo, h, wd = cfg["S"], cfg["f"], cfg["fo"], cfg["h"], cfg["w"]
    rng = np.random.default_rng(7)
    sel = np.unique(np.concatenate([[0, S * fo - 1], rng.integers(0, S * fo, 46)]))
    y = _np(hd.fft_conv_fprop(dx, dw)).reshape(S * fo, *[cfg["h"] - cfg["kh"] + 1] * 2)
    ref = oracle.conv_fprop(x, w, sel)
    assert np.max(np.abs(y[sel] - ref)) / np.max(np.abs(ref)) <= TOL
    sel = np.unique(np.concatenate([[0, S * f - 1], rng.integers(0, S * f, 46)]))
    gx = _np(hd.fft_conv_bprop(dgy, dw, h, wd)).reshape(S * f, h, wd)
    ref = oracle.conv_bprop(gy, w, h, wd, sel)
    assert np.max(np.abs(gx[sel] - ref)) / np.max(np.abs(ref)) <= TOL
    sel = np.unique(np.concatenate([[0, fo * f - 1], rng.integers(0, fo * f, 200)]))
    gw = _np(hd.fft_conv_accgrad(dx, dgy)).reshape(fo * f, cfg["kh"], cfg["kw"])
    ref = oracle.conv_accgrad(x, gy, sel)
    assert np.max(np.abs(gw[sel] - ref)) / np.max(np.abs(ref)) <= TOL


def test_accgrad_scale_and_accumulate(hd):
    cfg = dict(S=4, f=3, fo=5, h=10, w=10, kh=3, kw=3)
    x, w, gy = synth.conv_inputs(seed=101, **cfg)
    ref = oracle.conv_accgrad(x, gy)
    gw0 = synth.uniform_pm1(102, 0, w.shape)
    g = _dev(gw0)
    hd.fft_conv_accgrad(_dev(x), _dev(gy), gw=g, scale=0.25, accumulate=True)
    assert _relerr(_np(g), gw0.astype(np.float64) + 0.25 * ref) <= TOL
    g = _dev(gw0)
    hd.fft_conv_accgrad(_dev(x), _dev(gy), gw=g, scale=-2.0, accumulate=False)
    assert _relerr(_np(g), -2.0 * ref) <= TOL


def test_caller_workspace_and_errors(hd, lib):
    import torch
    cfg = dict(S=2, f=3, fo=4, h=9, w=9, kh=3, kw=3)
    x, w, gy = synth.conv_inputs(seed=103, **cfg)
    need = hd.workspace_bytes(lib.FPROP, 2, 3, 4, 9, 9, 3, 3)
    assert need > 0
    ws = torch.empty(need // 4, device="cuda", dtype=torch.float32)
    y = hd.fft_conv_fprop(_dev(x), _dev(w), ws=ws)
    assert _relerr(_np(y), oracle.conv_fprop(x, w)) <= TOL
    with pytest.raises(lib.FFTConvError, match="workspace too small"):
        hd.fft_conv_fprop(_dev(x), _dev(w), ws=ws[: need // 8])
    with pytest.raises(lib.FFTConvError, match="unsupported"):
        hd.fft_conv_fprop(torch.zeros((1, 1, 200, 200), device="cuda"), torch.zeros((1, 1, 130, 130), device="cuda"))
    with pytest.raises(lib.FFTConvError, match="invalid"):
        hd.fft_conv_fprop(torch.zeros((1, 1, 4, 4), device="cuda"), torch.zeros((1, 1, 5, 5), device="cuda"),
                          y=torch.zeros((1, 1, 1, 1), device="cuda"))


def test_repeat_calls_are_deterministic(hd):
    import torch
    cfg = synth.CONV_CONFIGS["C1"]
    x, w, _ = synth.conv_inputs(seed=0, **cfg)
    dx, dw = _dev(x), _dev(w)
    a = hd.fft_conv_fprop(dx, dw).clone()
    b = hd.fft_conv_fprop(dx, dw)
    assert torch.equal(a, b)


# (the last two take the one-launch form of the two backward contractions, with ragged tiles:
# accGrad first when its reduction, S, is the longer one, else bprop first)
@pytest.mark.parametrize("cfg", [SMALL[3], SMALL[6], SMALL[9], dict(S=9, f=20, fo=12, h=16, w=16, kh=3, kw=3),
                                 dict(S=140, f=8, fo=12, h=8, w=8, kh=3, kw=3),
                                 dict(S=4, f=72, fo=68, h=9, w=9, kh=3, kw=3)],
                         ids=lambda c: "S{S}f{f}fo{fo}_{h}x{w}_k{kh}x{kw}".format(**c))
def test_fprop_save_and_backward(hd, cfg):
    """Transform reuse: fprop_save + backward must give what the three independent passes give
    (each checked against the oracle), including the gx-only / gw-only forms."""
    import torch
    x, w, gy = synth.conv_inputs(seed=104, **cfg)
    dx, dw, dgy = _dev(x), _dev(w), _dev(gy)
    dims = (cfg["S"], cfg["f"], cfg["fo"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
    saved = torch.empty(hd.saved_bytes(*dims) // 4, device="cuda", dtype=torch.float32)
    y = hd.fft_conv_fprop_save(dx, dw, saved)
    assert _relerr(_np(y), oracle.conv_fprop(x, w)) <= TOL
    args = (cfg["f"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
    gx, gw = hd.fft_conv_backward(dgy, saved, *args)
    ref_gx, ref_gw = oracle.conv_bprop(gy, w, cfg["h"], cfg["w"]), oracle.conv_accgrad(x, gy)
    assert _relerr(_np(gx), ref_gx) <= TOL
    assert _relerr(_np(gw), ref_gw) <= TOL
    gx2, none = hd.fft_conv_backward(dgy, saved, *args, want_gw=False)
    assert none is None and torch.equal(gx2, gx)
    none, gw2 = hd.fft_conv_backward(dgy, saved, *args, want_gx=False, scale=0.5)
    assert none is None and _relerr(_np(gw2), 0.5 * ref_gw) <= TOL


@pytest.mark.parametrize("named", [False, True], ids=["library_basis", "named_basis"])
def test_reuse_at_c2(hd, named):
    """The step bench.py times: fprop_save + backward of the headline layer, on the basis the
    benchmark definition names (32, the launch configuration of `value`) and on the library's."""
    import torch
    cfg = {k: v for k, v in synth.CONV_CONFIGS["C2"].items() if k not in ("passes", "N")}
    x, w, gy = synth.conv_inputs(seed=synth.CONV_SEEDS["C2"], **cfg)
    dims = (cfg["S"], cfg["f"], cfg["fo"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
    if named:
        n = synth.CONV_CONFIGS["C2"]["N"]
        saved = torch.empty(hd.saved_bytes_tiled(*dims, n) // 4, device="cuda", dtype=torch.float32)
        y = hd.fft_conv_fprop_save_tiled(_dev(x), _dev(w), n, saved)
        gx, gw = hd.fft_conv_backward_tiled(_dev(gy), saved, cfg["f"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"], n)
    else:
        saved = torch.empty(hd.saved_bytes(*dims) // 4, device="cuda", dtype=torch.float32)
        y = hd.fft_conv_fprop_save(_dev(x), _dev(w), saved)
        gx, gw = hd.fft_conv_backward(_dev(gy), saved, cfg["f"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
    assert _relerr(_np(y), oracle.conv_fprop(x, w)) <= TOL
    assert _relerr(_np(gx), oracle.conv_bprop(gy, w, cfg["h"], cfg["w"])) <= TOL
    assert _relerr(_np(gw), oracle.conv_accgrad(x, gy)) <= TOL


@pytest.mark.parametrize("name", ["C3", "C4"])
def test_reuse_equals_separate_passes_at_full_size(hd, name):
    """The two-call step at the full size of the larger configurations on the library's own
    basis (14 and 64; both backward contractions in one launch where that applies) against the
    three independent passes, which the tests above check against the oracle (the step on the
    named bases, which the benchmark times, is checked against the oracle itself in
    test_bench_step_against_oracle_at_full_size).  Same transforms and the same products; only the order in which a contraction
    sums over k may differ (a lone contraction may split the tiles of a short last round of
    workgroups over its waves), so the results agree to rounding, far inside the 1e-4 bound."""
    import torch
    cfg = {k: v for k, v in synth.CONV_CONFIGS[name].items() if k not in ("passes", "N")}
    x, w, gy = synth.conv_inputs(seed=synth.CONV_SEEDS[name], **cfg)
    dx, dw, dgy = _dev(x), _dev(w), _dev(gy)
    dims = (cfg["S"], cfg["f"], cfg["fo"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
    saved = torch.empty(hd.saved_bytes(*dims) // 4, device="cuda", dtype=torch.float32)
    y = hd.fft_conv_fprop_save(dx, dw, saved)
    gx, gw = hd.fft_conv_backward(dgy, saved, cfg["f"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])

    def close(a, b):
        return float((a - b).abs().max()) <= 2e-6 * float(b.abs().max())
    assert close(y, hd.fft_conv_fprop(dx, dw))
    assert close(gx, hd.fft_conv_bprop(dgy, dw, cfg["h"], cfg["w"]))
    assert close(gw, hd.fft_conv_accgrad(dx, dgy))


@pytest.mark.parametrize("name", ["C3", "C4"])
def test_bench_step_against_oracle_at_full_size(hd, name):
    """The launch configuration bench.py times, against the oracle: fft_conv_fprop_save_tiled +
    fft_conv_backward_tiled at full size on the Fourier basis the configuration names (16 for
    the 13x13 layer, 64 for the 64x64 one).  The 13x13 layer is compared over the whole of y, gx
    and gw; for the 64x64 layer the oracle evaluates a seeded sample of output planes, all pixels
    of each, first and last plane included (256 planes of y and of gx, 1024 of gw)."""
    import torch
    cfg = {k: v for k, v in synth.CONV_CONFIGS[name].items() if k not in ("passes", "N")}
    n = synth.CONV_CONFIGS[name]["N"]
    x, w, gy = synth.conv_inputs(seed=synth.CONV_SEEDS[name], **cfg)
    dx, dw, dgy = _dev(x), _dev(w), _dev(gy)
    S, f, fo, h, wd, kh, kw = (cfg[k] for k in ("S", "f", "fo", "h", "w", "kh", "kw"))
    saved = torch.empty(hd.saved_bytes_tiled(S, f, fo, h, wd, kh, kw, n) // 4, device="cuda", dtype=torch.float32)
    y = _np(hd.fft_conv_fprop_save_tiled(dx, dw, n, saved))
    gx, gw = hd.fft_conv_backward_tiled(dgy, saved, f, h, wd, kh, kw, n)
    gx, gw = _np(gx), _np(gw)
    if name == "C3":
        assert _relerr(y, oracle.conv_fprop(x, w)) <= TOL
        assert _relerr(gx, oracle.conv_bprop(gy, w, h, wd)) <= TOL
        assert _relerr(gw, oracle.conv_accgrad(x, gy)) <= TOL
        return
    rng = np.random.default_rng(11)

    def sample(planes, k):
        return np.unique(np.concatenate([[0, planes - 1], rng.choice(planes, size=k - 2, replace=False)]))
    sel = sample(S * fo, 256)
    assert _relerr(y.reshape(S * fo, h - kh + 1, wd - kw + 1)[sel], oracle.conv_fprop(x, w, sel)) <= TOL
    sel = sample(S * f, 256)
    assert _relerr(gx.reshape(S * f, h, wd)[sel], oracle.conv_bprop(gy, w, h, wd, sel)) <= TOL
    sel = sample(fo * f, 1024)
    assert _relerr(gw.reshape(fo * f, kh, kw)[sel], oracle.conv_accgrad(x, gy, sel)) <= TOL


def test_saved_buffer_too_small(hd, lib):
    import torch
    cfg = dict(S=2, f=3, fo=4, h=9, w=9, kh=3, kw=3)
    x, w, gy = synth.conv_inputs(seed=105, **cfg)
    need = hd.saved_bytes(2, 3, 4, 9, 9, 3, 3)
    assert need > 0
    small = torch.empty(need // 8, device="cuda", dtype=torch.float32)
    with pytest.raises(lib.FFTConvError, match="workspace too small"):
        hd.fft_conv_fprop_save(_dev(x), _dev(w), small)


@pytest.mark.parametrize("cfg", [dict(S=128, f=64, fo=64, h=27, w=27, kh=5, kw=5),      # basis 28, 64x64 tiles + split tail
                                 dict(S=70, f=32, fo=96, h=13, w=13, kh=3, kw=3),       # basis 14, ragged M
                                 dict(S=8, f=64, fo=32, h=8, w=8, kh=3, kw=3)])         # basis 8: 64 planes per tile
def test_contraction_addressing_paths_agree(hd, lib, cfg, monkeypatch):
    """The contraction splits its gather / store addresses into a uniform and a per-lane part
    when every strided index moves in whole plane tiles; the general index arithmetic must
    give bit-identical results (same loads, same order of summation)."""
    import torch
    x, w, gy = synth.conv_inputs(seed=77, **cfg)
    dx, dw, dgy = (torch.from_numpy(a).cuda() for a in (x, w, gy))
    dims = (cfg["S"], cfg["f"], cfg["fo"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
    saved = torch.empty(hd.saved_bytes(*dims) // 4, device="cuda")

    def run(hd):
        y = hd.fft_conv_fprop_save(dx, dw, saved).clone()
        gx, gw = hd.fft_conv_backward(dgy, saved, cfg["f"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
        return y, gx.clone(), gw.clone(), hd.fft_conv_bprop(dgy, dw, cfg["h"], cfg["w"]).clone()
    fast = run(hd)
    monkeypatch.setenv("FFTCONV_GEMM_NO_FAST", "1")
    hd2 = lib.Handle(0)      # the switches are read from the environment when a handle is created
    try:
        general = run(hd2)
        torch.cuda.synchronize()
    finally:
        hd2.close()
    for a, b in zip(fast, general):
        assert torch.equal(a, b)
    ref = oracle.conv_fprop(x, w)
    assert np.max(np.abs(fast[0].cpu().numpy() - ref)) / np.max(np.abs(ref)) <= 1e-4


FUSED = [dict(S=16, f=16, fo=16, h=13, w=13, kh=3, kw=3),      # the smallest benchmark layer (basis 14)
         dict(S=5, f=4, fo=7, h=16, w=16, kh=5, kw=5),         # basis 16, padded LDS rows, ragged f'
         dict(S=3, f=32, fo=8, h=12, w=11, kh=2, kw=4),        # basis 12, f fills the plane tile
         dict(S=7, f=8, fo=3, h=8, w=8, kh=3, kw=3),           # basis 8 (64 planes per tile)
         dict(S=1, f=8, fo=32, h=14, w=13, kh=1, kw=1)]  # non-square image on a square basis


@pytest.mark.parametrize("cfg", FUSED, ids=lambda c: "S{S}f{f}fo{fo}_{h}x{w}_k{kh}x{kw}".format(**c))
def test_fused_fprop(hd, lib, cfg):
    """The one-launch fprop of small layers against the oracle and against the three-launch path."""
    import torch
    x, w, _ = synth.conv_inputs(seed=88, **cfg)
    dx, dw = _dev(x), _dev(w)
    wf = hd.fft_conv_transform_weights(dw, cfg["h"], cfg["w"])
    y = hd.fft_conv_fprop_fused(dx, wf, cfg["fo"], cfg["kh"], cfg["kw"])
    torch.cuda.synchronize()
    ref = oracle.conv_fprop(x, w)
    assert _relerr(_np(y), ref) <= TOL
    y3 = hd.fft_conv_fprop(dx, dw)       # the three-launch path
    assert float((y - y3).abs().max()) <= 2e-5 * float(np.max(np.abs(ref)))


def test_weights_ahead_passes_take_one_launch_for_small_layers(hd):
    """fft_conv_fprop_weights / fft_conv_bprop_weights run the smallest benchmark layer as one
    launch by themselves (the profiling interface reports a single kernel, "fused"), with the
    oracle's result; a layer beyond the one-launch kernels' range keeps its three launches."""
    import torch
    cfg = {k: v for k, v in synth.CONV_CONFIGS["C1"].items() if k not in ("passes", "N")}
    x, w, gy = synth.conv_inputs(seed=synth.CONV_SEEDS["C1"], **cfg)
    dx, dw, dgy = _dev(x), _dev(w), _dev(gy)
    wf = hd.fft_conv_transform_weights(dw, cfg["h"], cfg["w"])
    hd.set_profiling(True)
    try:
        y = hd.fft_conv_fprop_weights(dx, wf, cfg["fo"], cfg["kh"], cfg["kw"])
        assert hd.last_kernel_labels() == ["fused"]
        gx = hd.fft_conv_bprop_weights(dgy, wf, cfg["f"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
        assert hd.last_kernel_labels() == ["fused"]
        big = dict(S=4, f=64, fo=64, h=13, w=13, kh=3, kw=3)
        xb, wb, _ = synth.conv_inputs(seed=91, **big)
        wfb = hd.fft_conv_transform_weights(_dev(wb), 13, 13)
        yb = hd.fft_conv_fprop_weights(_dev(xb), wfb, 64, 3, 3)
        assert hd.last_kernel_labels() == ["fft.a", "contraction", "ifft"]
    finally:
        hd.set_profiling(False)
    torch.cuda.synchronize()
    assert _relerr(_np(y), oracle.conv_fprop(x, w)) <= TOL
    assert _relerr(_np(gx), oracle.conv_bprop(gy, w, cfg["h"], cfg["w"])) <= TOL
    assert _relerr(_np(yb), oracle.conv_fprop(xb, wb)) <= TOL


@pytest.mark.parametrize("cfg", FUSED, ids=lambda c: "S{S}f{f}fo{fo}_{h}x{w}_k{kh}x{kw}".format(**c))
def test_fused_bprop(hd, lib, cfg):
    """The one-launch bprop of small layers against the oracle and against the three-launch path."""
    import torch
    _, w, gy = synth.conv_inputs(seed=89, **cfg)
    dgy, dw = _dev(gy), _dev(w)
    wf = hd.fft_conv_transform_weights(dw, cfg["h"], cfg["w"])
    args = (cfg["f"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
    gx = hd.fft_conv_bprop_fused(dgy, wf, *args)
    torch.cuda.synchronize()
    ref = oracle.conv_bprop(gy, w, cfg["h"], cfg["w"])
    assert gx.shape == ref.shape
    assert _relerr(_np(gx), ref) <= TOL
    gx3 = hd.fft_conv_bprop(dgy, dw, cfg["h"], cfg["w"])       # the three-launch path
    assert float((gx - gx3).abs().max()) <= 2e-5 * float(np.max(np.abs(ref)))
    # a second call into the same output (stale LDS or output contents must not matter)
    gx.fill_(7.0)
    hd.fft_conv_bprop_fused(dgy, wf, *args, gx=gx)
    assert _relerr(_np(gx), ref) <= TOL


FUSED_ACC = [dict(S=16, f=16, fo=16, h=13, w=13, kh=3, kw=3),     # the smallest benchmark layer: 2 x 2 channel blocks
             dict(S=32, f=4, fo=4, h=14, w=14, kh=5, kw=5),       # a plane tile full of samples: one pair per workgroup
             dict(S=5, f=6, fo=9, h=12, w=11, kh=1, kw=1),        # 3 x 6 blocks: 18 pairs, padded to 32 lanes
             dict(S=3, f=16, fo=8, h=8, w=8, kh=3, kw=3),         # basis 8 (64 planes per tile)
             dict(S=64, f=3, fo=5, h=8, w=8, kh=8, kw=8),         # 64 samples on basis 8, kernel = image
             dict(S=7, f=10, fo=14, h=10, w=10, kh=3, kw=3),      # basis 10, odd sample count
             dict(S=2, f=64, fo=64, h=13, w=13, kh=3, kw=3)]      # 128 blocks of 4 x 8 channels


@pytest.mark.parametrize("cfg", FUSED_ACC, ids=lambda c: "S{S}f{f}fo{fo}_{h}x{w}_k{kh}x{kw}".format(**c))
def test_fused_accgrad(hd, lib, cfg):
    """The one-launch accGrad of small layers against the oracle and against the three-launch path
    (the same basis named through the tiled entry point, which never takes the one-launch kernel),
    with scale and accumulate, and into an output that holds stale values."""
    import torch
    x, _, gy = synth.conv_inputs(seed=90, **cfg)
    dx, dgy = _dev(x), _dev(gy)
    gw = hd.fft_conv_accgrad_fused(dx, dgy)
    torch.cuda.synchronize()
    ref = oracle.conv_accgrad(x, gy)
    assert gw.shape == ref.shape
    assert _relerr(_np(gw), ref) <= TOL
    n = hd.layer_basis(cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])[0]
    gw3 = hd.fft_conv_accgrad_tiled(dx, dgy, n)
    assert float((gw - gw3).abs().max()) <= 2e-5 * float(np.max(np.abs(ref)))
    gw.fill_(7.0)
    hd.fft_conv_accgrad_fused(dx, dgy, gw=gw)
    assert _relerr(_np(gw), ref) <= TOL
    acc = torch.full_like(gw, 1.5)
    hd.fft_conv_accgrad_fused(dx, dgy, gw=acc, scale=0.25, accumulate=True)
    assert _relerr(_np(acc), 1.5 + 0.25 * ref) <= TOL


def test_accgrad_takes_one_launch_for_few_samples(hd):
    """fft_conv_accgrad runs a layer of few samples as one launch by itself (the profiling
    interface reports a single kernel, "fused") with the oracle's result; the smallest benchmark
    layer, where three launches measured faster, keeps them."""
    import torch
    small = dict(S=2, f=32, fo=32, h=13, w=13, kh=3, kw=3)
    x, _, gy = synth.conv_inputs(seed=92, **small)
    c1 = {k: v for k, v in synth.CONV_CONFIGS["C1"].items() if k not in ("passes", "N")}
    x1, _, gy1 = synth.conv_inputs(seed=synth.CONV_SEEDS["C1"], **c1)
    hd.set_profiling(True)
    try:
        gw = hd.fft_conv_accgrad(_dev(x), _dev(gy))
        assert hd.last_kernel_labels() == ["fused"]
        gw1 = hd.fft_conv_accgrad(_dev(x1), _dev(gy1))
        assert hd.last_kernel_labels() == ["fft.ab", "contraction", "ifft"]
    finally:
        hd.set_profiling(False)
    torch.cuda.synchronize()
    assert _relerr(_np(gw), oracle.conv_accgrad(x, gy)) <= TOL
    assert _relerr(_np(gw1), oracle.conv_accgrad(x1, gy1)) <= TOL


def test_fused_accgrad_unsupported_shapes(hd, lib):
    import torch
    for cfg in (dict(S=33, f=4, fo=4, h=13, w=13, kh=3, kw=3),     # more samples than a plane tile holds
                dict(S=32, f=32, fo=32, h=13, w=13, kh=3, kw=3),   # 1024 single-pair blocks
                dict(S=2, f=16, fo=16, h=27, w=27, kh=5, kw=5),    # basis 28
                dict(S=2, f=8, fo=8, h=14, w=9, kh=1, kw=1)):      # rectangular basis 14 x 10
        x = torch.zeros((cfg["S"], cfg["f"], cfg["h"], cfg["w"]), device="cuda")
        gy = torch.zeros((cfg["S"], cfg["fo"], cfg["h"] - cfg["kh"] + 1, cfg["w"] - cfg["kw"] + 1), device="cuda")
        with pytest.raises(lib.FFTConvError, match="unsupported"):
            hd.fft_conv_accgrad_fused(x, gy)


def test_fused_fprop_unsupported_shapes(hd, lib):
    import torch
    for cfg in (dict(S=2, f=12, fo=8, h=13, w=13, kh=3, kw=3),     # f does not divide the plane tile
                dict(S=2, f=16, fo=40, h=13, w=13, kh=3, kw=3),    # f' beyond one plane tile
                dict(S=2, f=32, fo=32, h=13, w=13, kh=3, kw=3),    # more than 256 weight planes
                dict(S=2, f=16, fo=16, h=27, w=27, kh=5, kw=5),    # basis 28
                dict(S=1, f=8, fo=32, h=14, w=9, kh=1, kw=1)):     # rectangular basis 14 x 12
        x = torch.zeros((cfg["S"], cfg["f"], cfg["h"], cfg["w"]), device="cuda")
        w = torch.zeros((cfg["fo"], cfg["f"], cfg["kh"], cfg["kw"]), device="cuda")
        wf = hd.fft_conv_transform_weights(w, cfg["h"], cfg["w"])
        with pytest.raises(lib.FFTConvError, match="unsupported"):
            hd.fft_conv_fprop_fused(x, wf, cfg["fo"], cfg["kh"], cfg["kw"])
        gy = torch.zeros((cfg["S"], cfg["fo"], cfg["h"] - cfg["kh"] + 1, cfg["w"] - cfg["kw"] + 1), device="cuda")
        with pytest.raises(lib.FFTConvError, match="unsupported"):
            hd.fft_conv_bprop_fused(gy, wf, cfg["f"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
