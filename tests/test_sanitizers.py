"""AddressSanitizer + UndefinedBehaviorSanitizer over the CPU oracle and the library's host
control plane (pool_index.hpp): tests/sanitize_driver.cc runs both through seeded random call
sequences, compares their answers and lets the sanitizers watch every access.  CPU only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_and_host_control_plane_under_asan_ubsan(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("g++ not available")
    exe = str(tmp_path / "sanitize_driver")
    # the sanitizer runtime is linked statically: it must come first in the process, and the
    # environment may preload other libraries
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-Wall", "-Wextra",
           os.path.join(ROOT, "tests", "sanitize_driver.cc"),
           os.path.join(ROOT, "oracle", "mempool_oracle.cc"), "-o", exe]
    subprocess.check_call(cmd)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    out = subprocess.run([exe, "40"], capture_output=True, text=True, env=env, timeout=300)
    assert out.returncode == 0 and "sanitize ok" in out.stdout, out.stdout[-2000:] + out.stderr[-4000:]
