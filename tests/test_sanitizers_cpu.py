"""AddressSanitizer + UndefinedBehaviorSanitizer runs of the code that executes on the host: the C oracle, and the
host side of the C ABI (argument checks, layout / workspace arithmetic, state bookkeeping) with the kernel launchers
replaced by stubs.  No GPU is touched; GPU code is not instrumented (the sanitizer flags go to the host pass only)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="2")
ENV.pop("LD_PRELOAD", None)   # the sanitizer runtime has to come first in the driver's own process


def run_clean(exe):
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=300)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), (r.returncode, r.stdout[-2000:], r.stderr[-4000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-ffp-contract=off", "-fno-fast-math", "-fopenmp"] + SAN + [
        os.path.join(ROOT, "oracle", "pk_oracle.c"), os.path.join(HERE, "oracle_driver.c"), "-o", exe, "-lm"]
    subprocess.run(cmd, check=True)
    run_clean(exe)


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="no hipcc")
def test_api_host_checks_under_asan_ubsan(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    exe = str(tmp_path / "api_san")
    host_san = []
    for f in SAN[:2]:
        host_san += ["-Xarch_host", f]
    cmd = [hipcc, "-std=c++17", "--offload-arch=gfx950", "-O1", "-g", "-fno-omit-frame-pointer"] + host_san + [
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2510_05176_amd", "csrc"),
        os.path.join(ROOT, "paper_2510_05176_amd", "csrc", "pk_api.hip"), os.path.join(HERE, "api_driver.cpp"),
        "-x", "hip", "-o", exe]
    # api_driver.cpp includes a HIP header: compile it as HIP too
    cmd = [c for c in cmd if c not in ("-x", "hip")]
    cmd.insert(1, "-x")
    cmd.insert(2, "hip")
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-4000:]
    run_clean(exe)
