"""The row-group kernel's plan (groups, step and tile lists, per-m workgroup tables) checked on the host: the
driver builds them with the library's own code for hundreds of patterns and verifies every index the kernel
will follow.  No GPU needed; compiles one source file (a few seconds)."""
import os
import shutil
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_group_plan_is_consistent(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    exe = str(tmp_path / "host_group_plan_driver")
    csrc = os.path.join(ROOT, "paper_2007_13055_amd", "csrc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument", "-I", os.path.join(ROOT, "include"), "-I", csrc,
           os.path.join(ROOT, "tests", "host_group_plan_driver.cpp"), os.path.join(csrc, "bsr_mfma_group.hip"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, timeout=600)
    out = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "all consistent" in out.stdout
