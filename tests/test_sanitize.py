"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU).

oracle/oracle.c and the plain-C pins of tests/sanitize/oracle_pins.c are compiled with
-fsanitize=address,undefined and run; any access outside a buffer, signed overflow or misuse of
the heap in the oracle's index arithmetic aborts the program."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_oracle_pins_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_pins_san")
    subprocess.check_call(
        ["gcc", "-std=c99", "-O1", "-g", "-fno-omit-frame-pointer", "-fopenmp",
         "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-Wall",
         os.path.join(HERE, "sanitize", "oracle_pins.c"), os.path.join(ROOT, "oracle", "oracle.c"),
         "-o", exe, "-lm"])
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0"
    env["OMP_NUM_THREADS"] = "4"
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    print(run.stdout, run.stderr)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "all checks passed" in run.stdout
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr
