"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer: every routine, small random inputs and
edge cases, in a stand-alone binary (tests/sanitize/oracle_driver.c) with the sanitizer runtime linked in statically,
so that no library has to be preloaded."""
import os
import pathlib
import shutil
import subprocess

import pytest

ROOT = pathlib.Path(__file__).resolve().parent.parent
DRIVER = ROOT / "tests" / "sanitize" / "oracle_driver.c"
ORACLE = ROOT / "oracle" / "dessert_oracle.c"


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    exe = tmp_path / "oracle_sanitized"
    build = subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined",
                            "-static-libasan", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-Wall", "-Wextra",
                            str(ORACLE), str(DRIVER), "-o", str(exe), "-lm"], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    run = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300,
                         env=dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
                                  UBSAN_OPTIONS="print_stacktrace=1"))
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-4000:]
    assert "oracle sanitizer run: ok" in run.stdout
