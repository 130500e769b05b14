"""The library's host code (argument checks of every entry point in csrc/moe_api.hip, the expert planner in
csrc/plan.hip) built with AddressSanitizer and UndefinedBehaviorSanitizer on the host side and run through
tests/host_sanitizer_driver.cpp. The kernels are not in this build (the driver links stand-ins for their launchers:
every call it makes must be refused before a launcher is reached), so no GPU is needed."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2504_02263_amd", "csrc")


def test_host_code_is_clean_under_asan_and_ubsan():
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    out_dir = os.path.join(ROOT, "_build", "san")
    os.makedirs(out_dir, exist_ok=True)
    exe = os.path.join(out_dir, "host_san")
    cmd = [hipcc, "--offload-arch=gfx950", "-x", "hip", "-O1", "-g", "-std=c++17", "-w",
           "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           os.path.join(CSRC, "moe_api.hip"), os.path.join(CSRC, "plan.hip"),
           os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"), "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert build.returncode == 0, build.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    log = run.stdout + run.stderr
    assert run.returncode == 0, log[-3000:]
    assert "host checks done" in run.stdout
    assert "AddressSanitizer" not in log and "runtime error" not in log and "FAILED" not in log, log[-3000:]
