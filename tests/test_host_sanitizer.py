"""The plan builder under AddressSanitizer / UndefinedBehaviorSanitizer (host code only; no GPU needed).
Slow (the driver links every kernel, about 2.5 minutes), so it runs only when BSR_RUN_SANITIZER=1."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(os.environ.get("BSR_RUN_SANITIZER") != "1", reason="set BSR_RUN_SANITIZER=1 to build and run the sanitizer driver")
def test_plan_builder_under_sanitizers(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    exe = str(tmp_path / "host_sanitizer_driver")
    srcs = sorted(os.path.join(ROOT, "paper_2007_13055_amd", "csrc", f)
                  for f in os.listdir(os.path.join(ROOT, "paper_2007_13055_amd", "csrc")) if f.endswith(".hip"))
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
           "-fsanitize=undefined", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument", "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(ROOT, "paper_2007_13055_amd", "csrc"), os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"),
           *srcs, "-o", exe, "-fsanitize=address", "-fsanitize=undefined"]
    subprocess.run(cmd, check=True, capture_output=True, timeout=900)
    out = subprocess.run([exe], env=dict(os.environ, ASAN_OPTIONS="detect_leaks=0"), capture_output=True, text=True, timeout=600)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "no report" in out.stdout and "ERROR" not in out.stderr and "runtime error" not in out.stderr
