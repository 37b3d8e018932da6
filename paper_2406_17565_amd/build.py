"""Compile libmempool.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmempool.so")
SOURCES = ["kv_copy.hip", "block_hash.hip", "index_probe.hip", "mempool_api.hip"]
HEADERS = ["kv_copy.hpp", "pool_index.hpp", os.path.join("..", "..", "include", "mempool.h")]


def _hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: libmempool.so cannot be built")


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build(force: bool = True) -> str:
    if not force and not stale():
        return LIB
    cmd = [_hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-Wno-unused-parameter",
           # keep packed-FP32 instruction selection off for every kernel in this library
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    cmd += [os.path.join(CSRC, f) for f in SOURCES] + ["-o", LIB]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build())
