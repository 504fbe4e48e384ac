"""The host planner (tc_host.cpp: validation, schedule, tail split, model, inspection calls) built for the CPU with
AddressSanitizer and UndefinedBehaviorSanitizer and driven through the C ABI on host-only plans.  The device entry
points are replaced by stubs that fail (tests/host/device_stub.cpp); no GPU code runs."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_planner_under_asan_and_ubsan(tmp_path):
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no host C++ compiler")
    exe = str(tmp_path / "planner_driver")
    src = [os.path.join(ROOT, "paper_1704_03092_amd", "csrc", "tc_host.cpp"), os.path.join(ROOT, "tests", "host", "device_stub.cpp"),
           os.path.join(ROOT, "tests", "host", "planner_driver.cpp")]
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan", "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "paper_1704_03092_amd", "csrc"),
           "-o", exe] + src
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-6000:])
    assert "all checks passed" in run.stdout
