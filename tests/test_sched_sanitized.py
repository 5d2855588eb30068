"""The scheduler's host code under AddressSanitizer and UndefinedBehaviorSanitizer: the driver beside
this file calls every hat_sched_* entry point with valid and invalid arguments (CPU only)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_sched_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "sched_san")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "sched_sanitizer_driver.cpp"),
           os.path.join(ROOT, "paper_2503_18989_amd", "csrc", "sched.cpp"), "-o", exe]
    b = subprocess.run(cmd, capture_output=True, text=True)
    assert b.returncode == 0, b.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sched sanitizer driver: ok" in r.stdout and "runtime error" not in r.stderr


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_step_planner_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    """api.hip's host side (validation, pages, plan, work lists) through a host-only handle, with the
    sanitizers on the host code only; the driver stubs the kernels' launch functions."""
    exe = str(tmp_path / "planner_san")
    cmd = ["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all",
           os.path.join(ROOT, "paper_2503_18989_amd", "csrc", "api.hip"),
           os.path.join(ROOT, "tests", "planner_sanitizer_driver.hip"), "-o", exe]
    b = subprocess.run(cmd, capture_output=True, text=True)
    assert b.returncode == 0, b.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr[-3000:]
    assert "planner sanitizer driver: ok" in r.stdout and "runtime error" not in r.stderr
