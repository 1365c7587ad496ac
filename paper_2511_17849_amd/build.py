"""Builds libpier.so (HIP, gfx950) in-tree with hipcc.  Run as a script or call build()."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpier.so")
SOURCES = ["pier_kernels.hip", "pier_api.hip", "pier_placement.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    # keep hipcc from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # IEEE-correct fp32 division and square root on the device (the update rules are
    # stated with exact operations; the kernels also switch FMA contraction off)
    "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def build(verbose=False):
    cmd = [HIPCC, *FLAGS, "-o", LIB, *[os.path.join(CSRC, s) for s in SOURCES]]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


def build_abi_client(verbose=False):
    """The plain C-ABI client used by the GPU tests (tests/abi_client): links libpier.so,
    uses no torch."""
    root = os.path.dirname(HERE)
    src = os.path.join(root, "tests", "abi_client", "pier_client.cpp")
    exe = os.path.join(root, "tests", "abi_client", "pier_client")
    cmd = [HIPCC, "-O2", "-std=c++17", "--offload-arch=gfx950", "-o", exe, src,
           "-L" + HERE, "-lpier", "-Wl,-rpath,$ORIGIN/../../paper_2511_17849_amd"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return exe


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_abi_client(verbose=True))
    sys.exit(0)
