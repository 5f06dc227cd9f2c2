"""The host side of the C ABI (descriptor resolution, workspace layout, every reject path) compiled with
AddressSanitizer and UndefinedBehaviorSanitizer and run without a GPU: tests/host_sanitize/main.hip links
api.hip against stub launchers, so no kernel is launched.  A sanitizer report or a failed expectation
fails the test."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_validation_layer_under_asan_and_ubsan(tmp_path):
    hipcc = next((c for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", shutil.which("hipcc")) if c and os.path.exists(c)), None)
    if hipcc is None:
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "host_sanitize")
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-gpu-sanitize",
           "-fno-sanitize-recover=undefined", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2505_20776_amd", "csrc"),
           os.path.join(ROOT, "tests", "host_sanitize", "main.hip"),
           os.path.join(ROOT, "paper_2505_20776_amd", "csrc", "api.hip"), "-o", exe]
    build = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert build.returncode == 0, build.stdout[-4000:]
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert run.returncode == 0 and "all expectations held" in run.stdout, run.stdout[-4000:]
    assert "Sanitizer" not in run.stdout and "runtime error" not in run.stdout, run.stdout[-4000:]
