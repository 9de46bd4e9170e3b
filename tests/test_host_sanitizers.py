"""The host-only half of the C ABI (handle registry, block manager, prefix index, n-gram table,
combination selection) built HIP-free with g++ under AddressSanitizer + UndefinedBehaviorSanitizer
and driven through misuse (double free, use after free, foreign pointers) and random traces by
tests/host_asan_driver.cpp.  A sanitizer report aborts the driver; a wrong answer makes it exit 1."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_10380_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host C++ compiler")
def test_host_abi_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "host_asan_driver")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-Wall",
           os.path.join(ROOT, "tests", "host_asan_driver.cpp"), os.path.join(CSRC, "ax_host.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    assert "all checks passed" in r.stdout
