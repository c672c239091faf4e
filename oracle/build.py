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


def build(force: bool = False, sanitize: bool = False) -> str:
    out = LIB if not sanitize else os.path.join(HERE, "libllc_ref_asan.so")
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
        return out
    cmd = ["g++", "-std=c++17", "-O2", "-fno-fast-math", "-ffp-contract=off", "-fopenmp",
           "-shared", "-fPIC", "-Wall", "-Wextra", SRC, "-o", out]
    if sanitize:
        cmd[4:4] = ["-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer"]
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    print(build(force=True, sanitize="--asan" in sys.argv))
