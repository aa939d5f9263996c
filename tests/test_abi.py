"""The C-ABI library loads on a CPU-only host and exports every symbol the header declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "fftconv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(fft\w+)\s*\(", text)
    return sorted(set(n for n in names if not n.endswith("_handle")))


def test_header_symbols_exported():
    import paper_1412_7580_amd as pkg
    lib = pkg.load_library()
    decl = _declared()
    assert len(decl) >= 18
    for name in decl:
        assert hasattr(lib, name), f"{name} declared in fftconv.h but not exported"
    assert sorted(pkg.SYMBOLS) == decl


def test_host_only_calls():
    """Entry points that never touch the device: status strings and workspace sizing."""
    import paper_1412_7580_amd as pkg
    lib = pkg.load_library()
    assert lib.fftconv_status_string(0) == b"ok"
    assert b"workspace" in lib.fftconv_status_string(3)
    assert b"static" in lib.fftconv_status_string(5)
    assert lib.fftconv_static_scratch_bytes() == 32 << 20
    # fprop of the smallest configuration: 13x13 images take basis 14, so three frequency
    # tensors of 256 planes and 14 * 8 = 112 bins
    need = lib.fftconv_workspace_bytes(0, 16, 16, 16, 13, 13, 3, 3)
    assert need == 3 * 256 * 112 * 2 * 4
    assert lib.fftconv_saved_bytes(16, 16, 16, 13, 13, 3, 3) == 2 * 256 * 112 * 2 * 4
    # 16x16 images need basis 16 (144 bins); 27x27 take basis 28, whose 28 * 15 = 420 bins are
    # padded to 424 so that the bins split evenly over the eight XCDs
    assert lib.fftconv_workspace_bytes(0, 16, 16, 16, 16, 16, 3, 3) == 3 * 256 * 144 * 2 * 4
    assert lib.fftconv_workspace_bytes(0, 16, 16, 16, 27, 27, 5, 5) == 3 * 256 * 424 * 2 * 4
    # invalid (kernel larger than input, no such pass) and unsupported (kernel beyond every basis) shapes
    assert lib.fftconv_workspace_bytes(0, 1, 1, 1, 4, 4, 5, 5) == 0
    assert lib.fftconv_workspace_bytes(0, 1, 1, 1, 200, 200, 130, 130) == 0
    assert lib.fftconv_workspace_bytes(3, 1, 1, 1, 8, 8, 3, 3) == 0
    # an image beyond the largest basis is tiled: 200x200, 3x3 kernel -> the basis with the
    # fewest bins overall, and the same workspace as the explicit tiled call with that choice
    n = lib.fftconv_tile_basis(200, 200, 3, 3, 0)
    assert n in (8, 10, 12, 14, 16, 18, 20, 24, 28, 32, 36, 40, 48, 56, 64, 80, 96, 112, 128)
    assert lib.fftconv_workspace_bytes(0, 1, 1, 1, 200, 200, 3, 3) == \
        lib.fftconv_tiled_workspace_bytes(0, 1, 1, 1, 200, 200, 3, 3, n) > 0
    # forced basis 8 on a 20x20 image with a 3x3 kernel: 6x6 output tiles, 3x3 of them
    T = 64   # planes per workgroup at basis 8: buffers are padded to whole plane tiles
    pad = lambda planes: -(-planes // T) * T
    assert lib.fftconv_tiled_workspace_bytes(0, 2, 3, 4, 20, 20, 3, 3, 8) == \
        (pad(2 * 9 * 3) + pad(4 * 3) + pad(2 * 9 * 4)) * 40 * 2 * 4
    assert lib.fftconv_tiled_workspace_bytes(0, 2, 3, 4, 20, 20, 3, 3, 22) == 0   # no such basis
    assert lib.fftconv_tile_basis(20, 20, 9, 9, 8) == 0


def test_layer_basis_on_the_host():
    """Which basis the ordinary entry points take: square for square images, one size per side
    for other images whose sides both fit 32, tiles beyond the largest basis."""
    import ctypes
    import paper_1412_7580_amd as pkg
    lib = pkg.load_library()

    def basis(h, w, kh, kw, ph=0, pw=0):
        nr, nc = ctypes.c_int(-1), ctypes.c_int(-1)
        rc = lib.fftconv_layer_basis(h, w, kh, kw, ph, pw, ctypes.byref(nr), ctypes.byref(nc))
        return rc, nr.value, nc.value

    assert basis(13, 13, 3, 3) == (0, 14, 14)
    assert basis(27, 27, 5, 5) == (0, 28, 28)
    assert basis(27, 13, 5, 3) == (0, 28, 14)
    assert basis(8, 32, 3, 3) == (0, 8, 32)
    assert basis(40, 30, 9, 9) == (0, 40, 40)            # a side beyond 32: square
    assert basis(13, 27, 3, 3, 1, 1)[0] == 1             # margin padding: windows on a square basis
    rc, nr, nc = basis(200, 200, 3, 3)
    assert rc == 1 and nr == nc == lib.fftconv_tile_basis(200, 200, 3, 3, 0)
    assert basis(4, 4, 5, 5)[0] == -1                    # kernel larger than the image
    assert lib.fftconv_layer_basis(13, 13, 3, 3, 0, 0, None, None) == 0
    # 28 x 14 basis: 28 * 8 = 224 bins
    assert lib.fftconv_workspace_bytes(0, 16, 16, 16, 27, 13, 5, 3) == 3 * 256 * 224 * 2 * 4


def test_every_basis_is_accepted_by_name():
    """The nineteen Fourier bases: each can be named for an image it holds, sizes between them
    cannot, and the workspace of a named basis is three tensors of its bin count."""
    import paper_1412_7580_amd as pkg
    lib = pkg.load_library()
    bases = (8, 10, 12, 14, 16, 18, 20, 24, 28, 32, 36, 40, 48, 56, 64, 80, 96, 112, 128)
    tile = {8: 64, 10: 32, 12: 32, 14: 32, 16: 32, 18: 16, 20: 16, 24: 16, 28: 16, 32: 8, 36: 4, 40: 4, 48: 4, 56: 4,
            64: 4, 80: 1, 96: 1, 112: 1, 128: 1}
    for n in range(6, 130):
        got = lib.fftconv_tile_basis(n, n, 3, 3, n)
        assert got == (n if n in bases else 0), n
    for n in bases:
        unit = 32 if tile[n] == 4 else 8
        bins = -(-(n * (n // 2 + 1)) // unit) * unit
        planes = 64                                    # a multiple of every tile
        assert lib.fftconv_tiled_workspace_bytes(0, 8, 8, 8, n, n, 3, 3, n) == 3 * planes * bins * 2 * 4, n
    # an image takes the smallest basis that holds it
    import ctypes
    nr, nc = ctypes.c_int(), ctypes.c_int()
    untiled = 0
    for side in range(5, 129):
        tiled = lib.fftconv_layer_basis(side, side, 5, 5, 0, 0, ctypes.byref(nr), ctypes.byref(nc))
        assert tiled in (0, 1) and nr.value == nc.value and nr.value in bases
        if not tiled:                                   # (where tiles are estimated cheaper, any basis may come)
            untiled += 1
            assert nr.value == min(b for b in bases if b >= side), side
    assert untiled >= 50


def test_no_oracle_in_product():
    """The product package must not reach into the oracle."""
    pkg_dir = os.path.join(ROOT, "paper_1412_7580_amd")
    for dirpath, _, files in os.walk(pkg_dir):
        for fn in files:
            if fn.endswith((".py", ".hip", ".hpp", ".h")):
                src = open(os.path.join(dirpath, fn)).read()
                assert "import oracle" not in src and "from oracle" not in src and "liboracle" not in src
