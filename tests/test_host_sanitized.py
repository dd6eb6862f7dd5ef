"""The library's host side (planner, argument and call-order checks, tree tables, the per-level tables of a
drafting call, the verification-free step helpers) under AddressSanitizer and UndefinedBehaviorSanitizer on
the CPU: tests/host_fuzz.cpp replaces the HIP runtime and every kernel launcher by host stand-ins and drives
the complete call sequences with random valid and invalid inputs."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_side_is_clean_under_sanitizers(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None or not os.path.exists("/opt/rocm/include/hip/hip_runtime.h"):
        pytest.skip("needs g++ and the HIP headers")
    exe = str(tmp_path / "host_fuzz")
    cmd = [gxx, "-std=c++17", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(ROOT, "paper_2511_13587_amd", "csrc"), "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-static-libasan", "-g", "-O1", "-w",
           os.path.join(ROOT, "paper_2511_13587_amd", "csrc", "vvs_host.cpp"), os.path.join(ROOT, "tests", "host_fuzz.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    if r.returncode != 0 and "asan" in r.stderr.lower() and "cannot find" in r.stderr.lower():
        pytest.skip("the sanitizer runtime is not installed")
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0 and "host fuzz ok" in r.stdout, (r.stdout[-2000:], r.stderr[-3000:])
