"""fft_conv_fprop_static (the entry point that allocates nothing: its frequency-domain tensors
live in the library's static device array) against fft_conv_fprop, through the C ABI.

Two calls in a row on the same GPU, the second on a smaller layer, so that the second call finds
the first one's data in the array.  Bound as for every convolution parity test:
max|err| / max|ref| <= 1e-4, against the ordinary entry point and against the oracle."""
import numpy as np
import pytest

import oracle
from paper_1412_7580_amd import synth

pytestmark = pytest.mark.gpu
TOL = 1e-4


def _relerr(got, ref):
    return float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))


def test_static_scratch_fprop_matches_fprop(lib):
    import torch
    hd = lib.Handle(0)
    try:
        limit = hd.static_scratch_bytes()
        assert limit == 32 << 20
        # first a layer that uses most of the array (27x27 on basis 28: 424 bins), then a smaller
        # one on another basis (13x13 on basis 14), then the first again
        layers = [dict(S=16, f=64, fo=48, h=27, w=27, kh=5, kw=5),
                  dict(S=5, f=7, fo=3, h=13, w=13, kh=3, kw=3),
                  dict(S=16, f=64, fo=48, h=27, w=27, kh=5, kw=5)]
        for n, cfg in enumerate(layers):
            dims = (cfg["S"], cfg["f"], cfg["fo"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
            assert 0 < hd.workspace_bytes(lib.FPROP, *dims) <= limit
            x, w, _ = synth.conv_inputs(seed=300 + n, **cfg)
            dx, dw = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
            want = hd.fft_conv_fprop(dx, dw)
            got = torch.full_like(want, float("nan"))
            hd.fft_conv_fprop_static(dx, dw, got)
            torch.cuda.synchronize()
            g, r = got.cpu().numpy().astype(np.float64), want.cpu().numpy().astype(np.float64)
            assert np.isfinite(g).all(), cfg
            assert _relerr(g, r) <= TOL, (cfg, _relerr(g, r))
            assert _relerr(g, oracle.conv_fprop(x, w)) <= TOL, cfg
    finally:
        hd.close()


def test_static_scratch_rejects_large_layers(lib):
    import torch
    hd = lib.Handle(0)
    try:
        cfg = dict(S=128, f=64, fo=64, h=27, w=27, kh=5, kw=5)    # 78 MB of frequency-domain tensors
        assert hd.workspace_bytes(lib.FPROP, 128, 64, 64, 27, 27, 5, 5) > hd.static_scratch_bytes()
        x = torch.zeros((cfg["S"], cfg["f"], cfg["h"], cfg["w"]), device="cuda")
        w = torch.zeros((cfg["fo"], cfg["f"], cfg["kh"], cfg["kw"]), device="cuda")
        y = torch.full((cfg["S"], cfg["fo"], 23, 23), 7.0, device="cuda")
        with pytest.raises(lib.FFTConvError, match="static"):
            hd.fft_conv_fprop_static(x, w, y)
        torch.cuda.synchronize()
        assert bool((y == 7.0).all())      # nothing was launched
    finally:
        hd.close()
