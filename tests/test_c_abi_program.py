"""The library driven from plain C: tests/c_abi/check_passes.c includes include/fftconv.h as C99,
links libfftconv.so and the C oracle, and checks the passes, a tiled and a padded fprop, the
transform-reuse pair, the one-launch passes of a small layer and a 1-D transform on device buffers it allocates with the HIP runtime."""
import importlib.util
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def _builder():
    spec = importlib.util.spec_from_file_location("c_abi_build", os.path.join(HERE, "c_abi", "build.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_header_compiles_as_c99_and_program_links():
    """Every call the program makes must match the header's prototypes under a C compiler."""
    lib = os.path.join(os.path.dirname(HERE), "paper_1412_7580_amd", "libfftconv.so")
    if not os.path.exists(lib):
        pytest.skip("libfftconv.so not built")
    assert os.path.exists(_builder().build(force=True))


@pytest.mark.gpu
def test_plain_c_caller_matches_oracle():
    exe = _builder().build()
    env = dict(os.environ)
    env["LD_LIBRARY_PATH"] = os.pathsep.join(
        [os.path.join(os.path.dirname(HERE), "paper_1412_7580_amd"), env.get("LD_LIBRARY_PATH", "")])
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120, env=env)
    print(run.stdout, run.stderr)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "all checks passed" in run.stdout
    assert run.stdout.count("  ok\n") == 12
