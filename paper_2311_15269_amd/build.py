"""Builds the HIP library (gfx950) in-tree with hipcc."""
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libtessel_hip.so")
SOURCES = ["tessel_kernels.hip", "tessel_api.cpp"]
HEADERS = ["tessel_device.h", os.path.join("..", "..", "include", "tessel.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-x", "hip",
    # packed FP32 instructions are kept out of every device code object of this build
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # LDS and workspace words are read and written through pointers of several types (16-bit state next to 32-bit
    # tables, records as vectors and as words): no type-based alias analysis
    "-fno-strict-aliasing",
    "-Wall", "-Wno-unused-function",
]


def is_stale():
    if not os.path.exists(LIB):
        return True
    built = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > built for f in SOURCES + HEADERS)


def build_library(force=True, verbose=False):
    """hipcc --offload-arch=gfx950 ... -> paper_2311_15269_amd/libtessel_hip.so"""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + [os.path.join(CSRC, f) for f in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
