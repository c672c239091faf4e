"""Compile the CPU oracle (test infrastructure) into oracle/libllc_ref.so.

Plain g++; IEEE semantics are kept (-fno-fast-math) because the oracle's fp64
results are the reference the GPU path is compared against.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "llc_ref.cpp")
LIB = os.path.join(HERE, "libllc_ref.so")


def build(force: bool = False) -> str:
    """(The sanitizer build of the same source is tests/asan_driver.cpp, run by
    tests/test_oracle_sanitizers.py.)"""
    out = LIB
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
        return out
    cmd = ["g++", "-std=c++17", "-O2", "-fno-fast-math", "-ffp-contract=off", "-fopenmp",
           "-shared", "-fPIC", "-Wall", "-Wextra", SRC, "-o", out]
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    print(build(force=True))
