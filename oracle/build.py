"""Compile the CPU oracle into oracle/libflashoptim_oracle.so (test infrastructure only)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "flashoptim_oracle.cpp")
LIB = os.path.join(HERE, "libflashoptim_oracle.so")

# No fast-math, no FMA contraction: every operation is one rounded IEEE binary32 operation.
FLAGS = ["-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
         "-shared", "-fPIC", "-Wall", "-Wextra", "-Wno-misleading-indentation"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["g++"] + FLAGS + [SRC, "-o", LIB]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
