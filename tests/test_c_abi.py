"""The public header is valid C and the library can be driven from a plain C program."""
import os
import subprocess

import pytest

from paper_2406_17565_amd import build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXE = os.path.join(ROOT, "tests", "c_abi_smoke")


def _build():
    libdir = os.path.dirname(B.LIB)
    hip = "/opt/rocm/lib"
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c_abi_smoke.c"), "-o", EXE, "-L", libdir, "-lmempool",
           "-L", hip, "-lamdhip64", f"-Wl,-rpath,{libdir}", f"-Wl,-rpath,{hip}"]
    subprocess.check_call(cmd)


def test_header_compiles_as_c_and_host_calls_work():
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c",
                           os.path.join(ROOT, "include", "mempool.h")])
    _build()
    out = subprocess.run([EXE, "host"], capture_output=True, text=True)
    assert out.returncode == 0 and "host ok" in out.stdout, out.stdout + out.stderr


def test_per_request_bench_program_builds(tmp_path):
    """bench.py compiles bench_per_request.c at run time on the GPU machine: make sure it builds and
    links here (C99, warnings as errors), so a typo does not surface only there."""
    libdir, hip = os.path.dirname(B.LIB), "/opt/rocm/lib"
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "bench_per_request.c"), "-o", str(tmp_path / "bench_per_request"),
                           "-L", libdir, "-lmempool", "-L", hip, "-lamdhip64", f"-Wl,-rpath,{libdir}",
                           f"-Wl,-rpath,{hip}"])


@pytest.mark.gpu
def test_transfer_from_plain_c():
    if not os.path.exists(EXE):
        _build()
    out = subprocess.run([EXE, "gpu"], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0 and "gpu ok" in out.stdout, out.stdout + out.stderr
