"""Build the HIP library paper_1904_02205_amd/libpsb_hip.so for gfx950 (in-tree).

Usage: python -m paper_1904_02205_amd.build
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libpsb_hip.so")
SRC = os.path.join(HERE, "csrc", "psb_api.hip")
DEPS = [SRC,
        os.path.join(HERE, "csrc", "psb_kernels.hip.h"),
        os.path.join(HERE, "csrc", "psb_kernels_oc.hip.h"),
        os.path.join(HERE, "csrc", "psb_kernels_list.hip.h"),
        os.path.join(HERE, "csrc", "psb_kernels_shared.hip.h"),
        os.path.join(HERE, "csrc", "psb_kernels_glue.hip.h"),
        os.path.join(HERE, "csrc", "psb_philox.hip.h"),
        os.path.join(os.path.dirname(HERE), "include", "psb.h")]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         # packed FP32 instructions are disabled on purpose (see the build notes of this machine pool)
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-ffp-contract=off", "-Wall", "-Wno-unused-function"]


def source_id() -> str:
    """SHA-256 over the sources the library is built from, in the order of DEPS."""
    import hashlib
    h = hashlib.sha256()
    for d in DEPS:
        with open(d, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def build(verbose: bool = False, extra=()) -> str:
    cmd = ["hipcc", *FLAGS, f'-DPSB_BUILD_ID="{source_id()}"', *extra, SRC, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True, cwd=HERE)
    return LIB


def ensure_built() -> str:
    """Build only when the library is missing; a present library is used as it is."""
    if not os.path.exists(LIB):
        build()
    return LIB




if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
