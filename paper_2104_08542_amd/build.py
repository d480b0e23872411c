"""Builds libsfc.so (the C-ABI library of include/sfc.h) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "sfc_api.hip")
LIB = os.path.join(HERE, "libsfc.so")

FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-ffp-contract=off",            # optimizer arithmetic rounds like the plain formulas
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def build(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [hipcc] + FLAGS + os.environ.get("SFC_EXTRA_FLAGS", "").split() + [SRC, "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


EXAMPLE_SRC = os.path.join(HERE, "examples", "abi_client.cpp")
EXAMPLE_BIN = os.path.join(HERE, "examples", "abi_client")


def build_example(verbose=False):
    """The plain C++ client of the C ABI (no torch): links libsfc.so by path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    nopk = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    cmd = [hipcc, "-O2", "-std=c++17", "-ffp-contract=off", "--offload-arch=gfx950"] + nopk + [
           EXAMPLE_SRC, "-o", EXAMPLE_BIN, "-L" + HERE, "-lsfc", "-Wl,-rpath,$ORIGIN/.."]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    # the access-pattern ceilings that the kernel durations are read against
    cmd = [hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950"] + nopk + [os.path.join(HERE, "examples", "hbm_ceilings.hip"),
           "-o", os.path.join(HERE, "examples", "hbm_ceilings")]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return EXAMPLE_BIN


if __name__ == "__main__":
    build(verbose=True)
    build_example(verbose=True)
    print(LIB)
