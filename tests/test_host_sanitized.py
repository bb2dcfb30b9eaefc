"""The host code of the C ABI (csrc/api.hip: argument validation, workspace arithmetic, message formatting) under
AddressSanitizer and UndefinedBehaviorSanitizer.  api.hip is compiled again with the sanitizers on its host pass only
(the device pass and the other sources are the ordinary build's objects), linked into a library of its own, and
tests/sanitize/api_driver.c runs every path that needs no GPU against it."""
import os
import pathlib
import shutil
import subprocess

import pytest

ROOT = pathlib.Path(__file__).resolve().parent.parent
PKG = ROOT / "paper_2210_15748_amd"
DRIVER = ROOT / "tests" / "sanitize" / "api_driver.c"
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_c_abi_host_code_under_address_and_ub_sanitizers(tmp_path):
    from paper_2210_15748_amd import build as hip_build
    objs = [hip_build.OBJ / (s.rsplit(".", 1)[0] + ".o") for s in hip_build.SOURCES if s != "api.hip"]
    if not all(o.exists() for o in objs):
        hip_build.build(force=True)
    api_o = tmp_path / "api_san.o"
    lib = tmp_path / "libdessert_hip_san.so"
    exe = tmp_path / "api_sanitized"
    r = subprocess.run(["hipcc", *hip_build.FLAGS, *SAN, "-g", "-fno-omit-frame-pointer", "-c", str(PKG / "csrc" / "api.hip"),
                        "-o", str(api_o)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *SAN, "-shared-libsan", str(api_o), *map(str, objs),
                        "-o", str(lib)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    r = subprocess.run(["hipcc", "-x", "c", str(DRIVER), "-x", "none", *SAN, "-shared-libsan", "-g", "-L", str(tmp_path),
                        "-ldessert_hip_san", "-Wl,-rpath," + str(tmp_path), "-o", str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    rt = subprocess.run(["hipcc", "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True).stdout.strip()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    if rt and os.path.exists(rt):
        env["LD_LIBRARY_PATH"] = os.path.dirname(rt) + ":" + env.get("LD_LIBRARY_PATH", "")
    run = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300, env=env)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-4000:]
    assert "C ABI host sanitizer run: ok" in run.stdout
