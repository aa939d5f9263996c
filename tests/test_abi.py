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
    # fprop of the smallest configuration: three frequency tensors of 256 planes, 144 bins
    need = lib.fftconv_workspace_bytes(0, 16, 16, 16, 13, 13, 3, 3)
    assert need == 3 * 256 * 144 * 2 * 4
    assert lib.fftconv_saved_bytes(16, 16, 16, 13, 13, 3, 3) == 2 * 256 * 144 * 2 * 4
    # invalid (kernel larger than input) and unsupported (basis 256) shapes
    assert lib.fftconv_workspace_bytes(0, 1, 1, 1, 4, 4, 5, 5) == 0
    assert lib.fftconv_workspace_bytes(0, 1, 1, 1, 200, 200, 3, 3) == 0
    assert lib.fftconv_workspace_bytes(3, 1, 1, 1, 8, 8, 3, 3) == 0


def test_no_oracle_in_product():
    """The product package must not reach into the oracle."""
    pkg_dir = os.path.join(ROOT, "paper_1412_7580_amd")
    for dirpath, _, files in os.walk(pkg_dir):
        for fn in files:
            if fn.endswith((".py", ".hip", ".hpp", ".h")):
                src = open(os.path.join(dirpath, fn)).read()
                assert "import oracle" not in src and "from oracle" not in src and "liboracle" not in src
