"""Seeded random layer shapes through every form of the passes (ordinary, tiled with a random
valid basis, zero-padded), and through the transform-reuse pair in the same three forms, against
the time-domain oracle (GPU, C ABI).

The hand-picked cases of the other test files aim at known edges; this one sweeps the
combinations nobody thought of.  Bound: max|err| / max|ref| <= 1e-4 over each output tensor."""
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


def _draw(case):
    """Shape, mode and mode parameters of random case number `case`."""
    rng = np.random.default_rng(1000 + case)
    big = case % 5 == 0                                   # every fifth case: an image beyond basis 64
    h, w = (int(v) for v in rng.integers(65, 150, 2)) if big else (int(v) for v in rng.integers(3, 48, 2))
    kh, kw = int(rng.integers(1, min(h, 9) + 1)), int(rng.integers(1, min(w, 9) + 1))
    lim = 3 if big else 9
    S, f, fo = (int(v) for v in rng.integers(1, lim, 3))
    if case % 7 == 0:                                     # plane counts that allow 16-byte gathers
        S, f, fo = 4 * ((S + 3) // 4), 4 * ((f + 3) // 4), 4 * ((fo + 3) // 4)
    mode = ("ordinary", "tiled", "padded")[case % 3]
    cfg = dict(S=S, f=f, fo=fo, h=h, w=w, kh=kh, kw=kw)
    if mode == "tiled":
        bases = [n for n in (8, 10, 12, 14, 16, 18, 20, 24, 28, 32, 36, 40, 48, 56, 64) if n >= max(kh, kw)]
        return cfg, mode, (int(rng.choice(bases + [0])),)
    if mode == "padded":
        return cfg, mode, (int(rng.integers(0, 4)), int(rng.integers(0, 4)))
    return cfg, mode, ()


@pytest.mark.parametrize("case", range(60))
def test_random_shape(hd, case):
    cfg, mode, par = _draw(case)
    h, w = cfg["h"], cfg["w"]
    if mode == "padded":
        ph, pw = par
        big = dict(cfg, h=h + 2 * ph, w=w + 2 * pw)
        xp, wt, gy = synth.conv_inputs(seed=500 + case, **big)
        x = np.ascontiguousarray(xp[:, :, ph:ph + h, pw:pw + w])
        xpad = np.zeros_like(xp)
        xpad[:, :, ph:ph + h, pw:pw + w] = x
        dx, dw, dgy = _dev(x), _dev(wt), _dev(gy)
        got = (hd.fft_conv_fprop_padded(dx, dw, ph, pw), hd.fft_conv_bprop_padded(dgy, dw, h, w, ph, pw),
               hd.fft_conv_accgrad_padded(dx, dgy, ph, pw))
        ref = (oracle.conv_fprop(xpad, wt),
               oracle.conv_bprop(gy, wt, h + 2 * ph, w + 2 * pw)[:, :, ph:ph + h, pw:pw + w],
               oracle.conv_accgrad(xpad, gy))
    else:
        x, wt, gy = synth.conv_inputs(seed=500 + case, **cfg)
        dx, dw, dgy = _dev(x), _dev(wt), _dev(gy)
        if mode == "tiled":
            n = par[0]
            got = (hd.fft_conv_fprop_tiled(dx, dw, n), hd.fft_conv_bprop_tiled(dgy, dw, h, w, n),
                   hd.fft_conv_accgrad_tiled(dx, dgy, n))
        else:
            got = (hd.fft_conv_fprop(dx, dw), hd.fft_conv_bprop(dgy, dw, h, w), hd.fft_conv_accgrad(dx, dgy))
        ref = (oracle.conv_fprop(x, wt), oracle.conv_bprop(gy, wt, h, w), oracle.conv_accgrad(x, gy))
    for name, g, r in zip(("fprop", "bprop", "accgrad"), got, ref):
        e = _relerr(_np(g), r)
        assert e <= TOL, (name, cfg, mode, par, e)


def _draw_reuse(case):
    """Shape, mode and parameters of random case number `case` of the transform-reuse pair:
    channel counts in multiples of four (so that the backward pass pairs its contractions and,
    up to basis 32, its inverse transforms), every other image square."""
    rng = np.random.default_rng(2000 + case)
    h, w = (int(v) for v in rng.integers(4, 70, 2))
    if case % 2 == 0:
        w = h
    kh, kw = int(rng.integers(1, min(h, 7) + 1)), int(rng.integers(1, min(w, 7) + 1))
    S, f, fo = (4 * int(v) for v in rng.integers(1, 4, 3))
    if case % 5 == 0:
        S += 1
    cfg = dict(S=S, f=f, fo=fo, h=h, w=w, kh=kh, kw=kw)
    scale, acc = float(rng.choice([1.0, -0.5])), bool(rng.integers(0, 2))
    mode = ("ordinary", "tiled", "padded")[case % 3]
    if mode == "tiled":
        bases = [n for n in (8, 10, 12, 14, 16, 18, 20, 24, 28, 32, 36, 40, 48, 56, 64) if n >= max(kh, kw)]
        return cfg, mode, (int(rng.choice(bases)),), scale, acc
    if mode == "padded":
        return cfg, mode, (int(rng.integers(0, 3)), int(rng.integers(0, 3))), scale, acc
    return cfg, mode, (), scale, acc


@pytest.mark.parametrize("case", range(45))
def test_random_reuse_pair(hd, lib, case):
    """fft_conv_fprop_save + fft_conv_backward (ordinary, on a named basis, zero-padded) on random
    layers, with scale and accumulate on the weight gradients, against the oracle."""
    import torch
    cfg, mode, par, scale, acc = _draw_reuse(case)
    S, f, fo, h, w, kh, kw = (cfg[k] for k in ("S", "f", "fo", "h", "w", "kh", "kw"))
    dims = (S, f, fo, h, w, kh, kw)
    gw0 = torch.full((fo, f, kh, kw), 0.125, device="cuda")
    if mode == "padded":
        ph, pw = par
        xp, wt, gy = synth.conv_inputs(seed=700 + case, **dict(cfg, h=h + 2 * ph, w=w + 2 * pw))
        x = np.ascontiguousarray(xp[:, :, ph:ph + h, pw:pw + w])
        xpad = np.zeros_like(xp)
        xpad[:, :, ph:ph + h, pw:pw + w] = x
        dx, dw, dgy = _dev(x), _dev(wt), _dev(gy)
        saved = torch.empty(hd.saved_bytes_padded(*dims, ph, pw) // 4 + 1, device="cuda")
        y = hd.fft_conv_fprop_save_padded(dx, dw, ph, pw, saved)
        gx, gw = hd.fft_conv_backward_padded(dgy, saved, f, h, w, kh, kw, ph, pw, gw=gw0, scale=scale, accumulate=acc)
        ref = (oracle.conv_fprop(xpad, wt),
               oracle.conv_bprop(gy, wt, h + 2 * ph, w + 2 * pw)[:, :, ph:ph + h, pw:pw + w],
               oracle.conv_accgrad(xpad, gy))
    else:
        x, wt, gy = synth.conv_inputs(seed=700 + case, **cfg)
        dx, dw, dgy = _dev(x), _dev(wt), _dev(gy)
        if mode == "tiled":
            n = par[0]
            saved = torch.empty(hd.saved_bytes_tiled(*dims, n) // 4 + 1, device="cuda")
            y = hd.fft_conv_fprop_save_tiled(dx, dw, n, saved)
            gx, gw = hd.fft_conv_backward_tiled(dgy, saved, f, h, w, kh, kw, n, gw=gw0, scale=scale, accumulate=acc)
        else:
            saved = torch.empty(hd.saved_bytes(*dims) // 4 + 1, device="cuda")
            y = hd.fft_conv_fprop_save(dx, dw, saved)
            gx, gw = hd.fft_conv_backward(dgy, saved, f, h, w, kh, kw, gw=gw0, scale=scale, accumulate=acc)
        ref = (oracle.conv_fprop(x, wt), oracle.conv_bprop(gy, wt, h, w), oracle.conv_accgrad(x, gy))
    want_gw = scale * ref[2] + (0.125 if acc else 0.0)
    for name, g, r in zip(("fprop_save", "backward gx", "backward gw"), (y, gx, gw), (ref[0], ref[1], want_gw)):
        e = _relerr(_np(g), r)
        assert e <= TOL, (name, cfg, mode, par, scale, acc, e)
