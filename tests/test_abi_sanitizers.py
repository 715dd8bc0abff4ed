"""Host sanitizer build of the C ABI's argument-checking layer (csrc/api.hip), run on the CPU.

The layer is compiled with AddressSanitizer and UndefinedBehaviorSanitizer for the host pass only, linked
with stand-in launch functions into a small driver that makes calls which must all be refused before any
launch (tests/host_sanitize/).  A sanitizer report or a wrong status fails the test."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "host_sanitize")
BUILD = os.path.join(ROOT, "_build", "host_sanitize")


@pytest.mark.timeout(600)
def test_validation_layer_under_asan_and_ubsan():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    os.makedirs(BUILD, exist_ok=True)
    exe = os.path.join(BUILD, "abi_driver")
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fno-omit-frame-pointer",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
           os.path.join(ROOT, "paper_2409_09099_amd", "csrc", "api.hip"), os.path.join(SRC, "launch_stubs.cpp"),
           os.path.join(SRC, "abi_driver.cpp"), "-o", exe]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout[-4000:]
    assert "abi driver ok" in run.stdout and "runtime error" not in run.stdout and "AddressSanitizer" not in run.stdout, run.stdout[-4000:]
    shutil.rmtree(BUILD, ignore_errors=True)
