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


def build(force: bool = True, src: str = SRC, out: str = LIB) -> str:
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(src):
        return out
    cmd = ["g++"] + FLAGS + [src, "-o", out]
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
