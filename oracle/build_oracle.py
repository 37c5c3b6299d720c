"""Compile the CPU oracle (test infrastructure) into oracle/libpsb_oracle.so.

Usage: python oracle/build_oracle.py
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libpsb_oracle.so")
SRC = os.path.join(HERE, "psb_oracle.cpp")

# No fast-math and no contraction: the rescale must be four separately rounded
# binary32 operations.
FLAGS = ["-O2", "-std=c++17", "-fno-fast-math", "-ffp-contract=off", "-fopenmp",
         "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(verbose: bool = False) -> str:
    cmd = ["g++", *FLAGS, SRC, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True, cwd=HERE)
    return LIB


def ensure_built() -> str:
    """Build only when the library is missing or older than its sources."""
    srcs = [SRC, os.path.join(HERE, "psb_oracle.h")]
    if (not os.path.exists(LIB)) or any(os.path.getmtime(s) > os.path.getmtime(LIB) for s in srcs):
        build()
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
