"""Build tests/c_abi/check_passes: a plain-C program (gcc, C99) that calls the library through
include/fftconv.h and checks it against oracle/oracle.c.  Test infrastructure."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
BIN = os.path.join(HERE, "_build", "check_passes")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build(force: bool = False) -> str:
    src = [os.path.join(HERE, "check_passes.c"), os.path.join(ROOT, "oracle", "oracle.c")]
    lib_dir = os.path.join(ROOT, "paper_1412_7580_amd")
    newest = max(os.path.getmtime(p) for p in src + [os.path.join(ROOT, "include", "fftconv.h")])
    if force or not os.path.exists(BIN) or os.path.getmtime(BIN) < newest:
        os.makedirs(os.path.dirname(BIN), exist_ok=True)
        subprocess.check_call(
            ["gcc", "-std=c99", "-O2", "-fopenmp", "-Wall", "-Wno-unused-result", "-D_GNU_SOURCE",
             "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROCM, "include")] + src +
            ["-o", BIN, "-L" + lib_dir, "-lfftconv", "-L" + os.path.join(ROCM, "lib"), "-lamdhip64", "-lm",
             "-Wl,-rpath," + lib_dir, "-Wl,-rpath," + os.path.join(ROCM, "lib")])
    return BIN


if __name__ == "__main__":
    print(build(force=True))
