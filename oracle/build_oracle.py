"""Compile the CPU oracle (test infrastructure) into oracle/libpsb_oracle.so.

Usage: python oracle/build_oracle.py              build the library
       python oracle/build_oracle.py --sanitize   build the oracle and its check driver with -fsanitize=address,undefined
                                                  and run the driver (exit status 0 = nothing reported)
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


def sanitize(verbose: bool = False) -> int:
    """Build the oracle with its check driver under AddressSanitizer and UndefinedBehaviorSanitizer (host code only)
    and run it: every oracle entry point on small, exactly sized buffers.  Returns the driver's exit status."""
    exe = os.path.join(HERE, "sanitize_check")
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-fno-fast-math", "-ffp-contract=off", "-fopenmp",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-Wall", "-Wextra",
           SRC, os.path.join(HERE, "sanitize_check.cpp"), "-o", exe]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True, cwd=HERE)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    return subprocess.run([exe], env=env, cwd=HERE).returncode


def ensure_built() -> str:
    """Build only when the library is missing or older than its sources."""
    srcs = [SRC, os.path.join(HERE, "psb_oracle.h")]
    if (not os.path.exists(LIB)) or any(os.path.getmtime(s) > os.path.getmtime(LIB) for s in srcs):
        build()
    return LIB


if __name__ == "__main__":
    if "--sanitize" in sys.argv[1:]:
        sys.exit(sanitize(verbose=True))
    print(build(verbose=True))
    sys.exit(0)
