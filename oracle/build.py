"""Compile the CPU oracle (test infrastructure) into oracle/liboracle.so with g++."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "liboracle.so")


def build(force: bool = True) -> str:
    src = os.path.join(HERE, "mempool_oracle.cc")
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(src):
        return LIB
    cmd = ["g++", "-std=c++17", "-O2", "-Wall", "-Wextra", "-shared", "-fPIC", src, "-o", LIB]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build())
