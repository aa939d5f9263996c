"""The host-side planner (basis choice, tiling, window views, workspace layout) checked on the CPU.

fftconv_describe_plan() returns the plan of a pass as numbers.  For a grid of layer shapes
(square and non-square images and kernels, margin padding, named and library-chosen bases,
tiled and untiled) this test
  * asserts the structural invariants: every window and crop fits its transform, the tiles cover
    the output exactly, the workspace regions are aligned, ordered and large enough;
  * re-enacts the plan in numpy -- gather the windows the plan describes (zeros outside the
    image), transform on the plan's basis, contract with the plan's matrix sizes, strides and
    conjugates, invert, crop and scatter as the plan says -- and compares with the time-domain
    oracle (Section 2's equations; tiling as in Section 6).  This is what the kernels do with the
    plan, so a planner mistake shows here without a GPU.
"""
import itertools

import numpy as np
import pytest

import oracle
import paper_1412_7580_amd as pkg
from paper_1412_7580_amd import synth

BASES = (8, 10, 12, 14, 16, 18, 20, 24, 28, 32, 36, 40, 48, 56, 64, 80, 96, 112, 128)


def _gather(img, planes, hwin, wwin, view):
    """Operand planes [planes, hwin, wwin]: whole planes, or the windows of a view."""
    S, C, H, W = img.shape
    if not view["view"]:
        assert planes == S * C and (hwin, wwin) == (H, W)
        return img.reshape(planes, H, W).astype(np.float64)
    assert (view["C"], view["H"], view["W"]) == (C, H, W)
    out = np.zeros((planes, hwin, wwin))
    for p in range(planes):
        m, ch = divmod(p, C)
        q, tx = divmod(m, view["ntx"])
        s, ty = divmod(q, view["nty"])
        y0, x0 = ty * view["dy"] + view["oy"], tx * view["dx"] + view["ox"]
        for r in range(hwin):
            gy = y0 + r
            if not 0 <= gy < H:
                continue
            lo, hi = max(0, -x0), min(wwin, W - x0)
            if hi > lo:
                out[p, r, lo:hi] = img[s, ch, gy, x0 + lo:x0 + hi]
    return out


def _scatter(blocks, shape, hc, wc, view):
    """Result tensor from the crops [planes, >=hc, >=wc] of the inverse transforms."""
    S, C, H, W = shape
    if not view["view"]:
        return blocks[:, :hc, :wc].reshape(S, C, hc, wc)
    out = np.full(shape, np.nan)
    for p in range(blocks.shape[0]):
        m, ch = divmod(p, C)
        q, tx = divmod(m, view["ntx"])
        s, ty = divmod(q, view["nty"])
        y0, x0 = ty * view["dy"], tx * view["dx"]
        hh, ww = min(hc, H - y0), min(wc, W - x0)
        assert hh > 0 and ww > 0, "an empty tile"
        assert np.isnan(out[s, ch, y0:y0 + hh, x0:x0 + ww]).all(), "two tiles write one pixel"
        out[s, ch, y0:y0 + hh, x0:x0 + ww] = blocks[p, view["oy"]:view["oy"] + hh, view["ox"]:view["ox"] + ww]
    assert not np.isnan(out).any(), "a pixel no tile writes"
    return out


def _enact(pass_, x, w, gy, cfg, tile_n, ph, pw):
    S, f, fo, h, wd, kh, kw = (cfg[k] for k in ("S", "f", "fo", "h", "w", "kh", "kw"))
    d = pkg.describe_plan(pass_, S, f, fo, h, wd, kh, kw, tile_n, ph, pw)
    Nr, Nc = d["Nr"], d["Nc"]
    opA, opB = {pkg.FPROP: (x, w), pkg.BPROP: (gy, w), pkg.ACCGRAD: (gy, x)}[pass_]
    out_shape = {pkg.FPROP: gy.shape, pkg.BPROP: x.shape, pkg.ACCGRAD: w.shape}[pass_]
    # ---- invariants
    for hh, ww in ((d["hA"], d["wA"]), (d["hB"], d["wB"])):
        assert 0 < hh <= Nr and 0 < ww <= Nc, "a window larger than the transform"
    vC = d["C"]
    assert vC["oy"] + d["hC"] <= Nr and vC["ox"] + d["wC"] <= Nc, "the crop leaves the transform"
    assert d["bins"] >= Nr * (Nc // 2 + 1) and d["bins"] % 8 == 0
    T = 1 << d["tile_log2"]
    tile_bytes = lambda planes: -(-planes // T) * T * d["bins"] * 2 * 4
    assert d["bytesA"] == tile_bytes(d["planesA"])
    assert d["offA"] % 256 == 0 and d["offB"] % 256 == 0 and d["offC"] % 256 == 0 and d["total"] % 256 == 0
    assert d["offB"] >= d["offA"] + tile_bytes(d["planesA"])
    assert d["offC"] >= d["offB"] + tile_bytes(d["planesB"])
    assert d["total"] >= d["offC"] + tile_bytes(d["planesC"])
    M, N, K = d["M"], d["N"], d["K"]
    for rs, cs, rows, cols, planes in ((d["a_rs"], d["a_cs"], M, K, d["planesA"]),
                                       (d["b_rs"], d["b_cs"], K, N, d["planesB"]),
                                       (d["c_rs"], d["c_cs"], M, N, d["planesC"])):
        assert (rows - 1) * rs + (cols - 1) * cs == planes - 1, "matrix does not span its planes"
    # ---- re-enactment
    A = _gather(opA, d["planesA"], d["hA"], d["wA"], d["A"])
    B = _gather(opB, d["planesB"], d["hB"], d["wB"], d["B"])
    AF = np.fft.rfft2(A, s=(Nr, Nc))
    BF = np.fft.rfft2(B, s=(Nr, Nc))
    if d["conjA"]:
        AF = AF.conj()
    if d["conjB"]:
        BF = BF.conj()
    mi, ki, ni = np.arange(M), np.arange(K), np.arange(N)
    Am = AF[(mi[:, None] * d["a_rs"] + ki[None, :] * d["a_cs"])]        # [M, K, Nr, Nc/2+1]
    Bm = BF[(ki[:, None] * d["b_rs"] + ni[None, :] * d["b_cs"])]        # [K, N, ...]
    Cm = np.einsum("mkab,knab->mnab", Am, Bm)
    CF = np.empty((d["planesC"],) + Cm.shape[2:], dtype=complex)
    CF[(mi[:, None] * d["c_rs"] + ni[None, :] * d["c_cs"])] = Cm
    blocks = np.fft.irfft2(CF, s=(Nr, Nc))
    return _scatter(blocks, out_shape, d["hC"], d["wC"], vC), d


def _padded(x, ph, pw):
    return np.pad(x, ((0, 0), (0, 0), (ph, ph), (pw, pw)))


SHAPES = [
    # (S, f, fo, h, w, kh, kw, tile_n, ph, pw)
    (2, 3, 2, 13, 13, 3, 3, -1, 0, 0),      # library basis 14, untiled
    (2, 2, 3, 13, 13, 3, 3, 16, 0, 0),      # named basis holding the image
    (1, 2, 2, 27, 13, 5, 3, -1, 0, 0),      # rectangular basis 28 x 14
    (1, 2, 2, 20, 20, 3, 3, 8, 0, 0),       # tiled at 8: 6x6 output tiles, ragged last tiles
    (1, 2, 3, 23, 17, 4, 2, 10, 0, 0),      # non-square everything, tiled at 10
    (1, 1, 2, 40, 13, 3, 3, -1, 0, 0),      # strongly rectangular: the library tiles it
    (1, 2, 1, 9, 9, 3, 3, -1, 1, 1),        # margin padding, one window per image
    (2, 1, 2, 11, 8, 3, 5, -1, 2, 3),       # padding larger than one, non-square kernel
    (1, 2, 2, 19, 21, 5, 3, 12, 2, 1),      # padded and tiled
    (1, 1, 1, 12, 12, 12, 12, -1, 0, 0),    # kernel as large as the image
    (1, 2, 2, 16, 16, 1, 1, 8, 0, 0),       # 1x1 kernel: tiles do not overlap
    (1, 1, 1, 70, 70, 3, 3, 0, 0, 0),       # library's choice of tile basis
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "S{}f{}fo{}_{}x{}_k{}x{}_t{}_p{}x{}".format(*s))
def test_plan_reenacted_in_numpy_matches_oracle(shape):
    S, f, fo, h, w, kh, kw, tile_n, ph, pw = shape
    cfg = dict(S=S, f=f, fo=fo, h=h, w=w, kh=kh, kw=kw)
    rng = np.random.default_rng(5)
    x = rng.uniform(-1, 1, (S, f, h, w))
    wt = rng.uniform(-1, 1, (fo, f, kh, kw))
    hp, wp = h + 2 * ph, w + 2 * pw
    gy = rng.uniform(-1, 1, (S, fo, hp - kh + 1, wp - kw + 1))
    xp = _padded(x, ph, pw)
    ref = {pkg.FPROP: oracle.conv_fprop(xp, wt),
           pkg.BPROP: oracle.conv_bprop(gy, wt, hp, wp)[:, :, ph:ph + h, pw:pw + w],
           pkg.ACCGRAD: oracle.conv_accgrad(xp, gy)}
    for pass_ in (pkg.FPROP, pkg.BPROP, pkg.ACCGRAD):
        got, d = _enact(pass_, x, wt, gy, cfg, tile_n, ph, pw)
        err = np.max(np.abs(got - ref[pass_])) / np.max(np.abs(ref[pass_]))
        assert err <= 1e-10, (pass_, err, d)


def test_plan_invariants_over_a_shape_grid():
    """Every image size 1 ... 140 (square, and against three other widths) with kernels 1 ... 11 and
    paddings 0 ... 2, as the ordinary entry points plan them: sizes consistent, tiles cover the
    output, windows and crops inside the transform."""
    lib = pkg.load_library()
    checked = 0
    for h in list(range(1, 70)) + [96, 100, 127, 128, 129, 140]:
        for w in {h, max(1, h // 2), min(140, h + 7), 13}:
            for k, p in itertools.product((1, 2, 3, 5, 11), (0, 1, 2)):
                if k > h + 2 * p or k > w + 2 * p:
                    continue
                for pass_ in (pkg.FPROP, pkg.BPROP, pkg.ACCGRAD):
                    d = pkg.describe_plan(pass_, 2, 3, 4, h, w, k, k, -1, p, p)
                    N = d["Nr"]
                    assert d["Nr"] in BASES and d["Nc"] in BASES
                    oh, ow = h + 2 * p - k + 1, w + 2 * p - k + 1
                    if d["tiled"]:
                        dy = dx = N - k + 1
                        assert dy >= 1
                        ext = (h, w) if pass_ == pkg.BPROP else (oh, ow)
                        v = d["A"] if pass_ != pkg.FPROP else d["C"]
                        if pass_ == pkg.BPROP:
                            v = d["C"]
                        assert v["view"] and (v["dy"], v["dx"]) == (dy, dx)
                        assert (v["nty"] - 1) * dy < ext[0] <= v["nty"] * dy
                        assert (v["ntx"] - 1) * dx < ext[1] <= v["ntx"] * dx
                    else:
                        assert d["Nr"] >= h and d["Nc"] >= w and p == 0
                    assert d["C"]["oy"] + d["hC"] <= d["Nr"] and d["C"]["ox"] + d["wC"] <= d["Nc"]
                    assert d["hA"] <= d["Nr"] and d["wA"] <= d["Nc"] and d["hB"] <= d["Nr"] and d["wB"] <= d["Nc"]
                    assert d["total"] == lib.fftconv_padded_workspace_bytes(pass_, 2, 3, 4, h, w, k, k, p, p)
                    checked += 1
    assert checked > 5000


def test_describe_plan_rejects_bad_shapes():
    with pytest.raises(pkg.FFTConvError, match="invalid"):
        pkg.describe_plan(pkg.FPROP, 1, 1, 1, 4, 4, 5, 5)
    with pytest.raises(pkg.FFTConvError, match="invalid"):
        pkg.describe_plan(pkg.FPROP, 1, 1, 1, 20, 20, 3, 3, 22)      # 22 is not a basis
    with pytest.raises(pkg.FFTConvError, match="unsupported"):
        pkg.describe_plan(pkg.FPROP, 1, 1, 1, 200, 200, 130, 130)
