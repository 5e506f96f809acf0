"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer: oracle/mv_oracle.c is
compiled together with a small C driver (tests/oracle_sanitizer_driver.c) that calls every
entry point on exact-size buffers; a read or write outside an argument, a signed overflow
or a misaligned access anywhere in the oracle fails the run.  Host code only."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "mv_oracle.c")
DRIVER = os.path.join(ROOT, "tests", "oracle_sanitizer_driver.c")


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "oracle_sanitized")
    # the sanitizer runtimes linked statically: a preloaded library may then come first
    cmd = [gcc, "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-static-libasan", "-static-libubsan",
           "-Wall", "-Wextra", SRC, DRIVER, "-o", exe, "-lm"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and ("libasan" in built.stderr or "libubsan" in built.stderr):
        pytest.skip("sanitizer runtimes not installed: " + built.stderr.strip().splitlines()[-1])
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", OMP_NUM_THREADS="4")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    sys.stdout.write(run.stdout[-2000:])
    sys.stderr.write(run.stderr[-6000:])
    assert run.returncode == 0, "sanitizer report or failed check:\n" + run.stderr[-6000:]
    assert run.stdout.strip().endswith("ok")
