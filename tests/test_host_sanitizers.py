"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer (host side only; the
device code is compiled as usual and never runs here): builds a driver that links the library's sources
and walks every entry point's argument checks, workspace arithmetic and host-only functions with valid,
invalid and extreme arguments. Any sanitizer report or failed check fails the test."""
import glob
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.timeout(600)
def test_host_code_under_asan_and_ubsan(tmp_path):
    csrc = os.path.join(ROOT, "paper_2603_02631_amd", "csrc")
    srcs = sorted(glob.glob(os.path.join(csrc, "*.hip")) + glob.glob(os.path.join(csrc, "*.cpp")))
    exe = str(tmp_path / "sanitize_driver")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-fsanitize=address,undefined", "-fno-gpu-sanitize", "-fno-sanitize-recover=undefined",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Xarch_device", "-fno-honor-nans",
           "-I", os.path.join(ROOT, "include"), "-I", csrc,
           os.path.join(ROOT, "tests", "host", "sanitize_driver.cpp"), *srcs, "-o", exe]
    build = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert build.returncode == 0, build.stdout[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout[-4000:]
    assert "all checks passed" in run.stdout
    assert "runtime error" not in run.stdout and "AddressSanitizer" not in run.stdout
