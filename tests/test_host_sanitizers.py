"""The host layer of libkvs (argument validation, workspace carve-up, unit tables, launch sequencing) built with
AddressSanitizer and UndefinedBehaviorSanitizer on the CPU and driven through the C ABI by tests/host/abi_driver.cpp.
The kernel launchers are replaced by stubs (tests/host/launch_stubs.cpp) that check the tables they are handed, so
whole calls on problems of up to 150 ragged units run to their end without a GPU."""

import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOST = os.path.join(ROOT, "tests", "host")
CSRC = os.path.join(ROOT, "paper_2603_00907_amd", "csrc")


def test_host_layer_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    hipcc = "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not installed")
    exe = str(tmp_path / "abi_driver")
    # sanitizers on the host pass only (each -fsanitize= directly after -Xarch_host); the device pass of
    # kvs_api.hip holds nothing but the static scratch array
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-x", "hip"] + san + [
        "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
        os.path.join(CSRC, "kvs_api.hip"), os.path.join(HOST, "launch_stubs.cpp"), os.path.join(HOST, "abi_driver.cpp"),
        "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, (run.stdout[-3000:], run.stderr[-3000:])
    assert "all checks passed" in run.stdout
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr
