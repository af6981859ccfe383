"""Builds libdynadiag.so (the HIP kernels plus the C ABI) for gfx950 with hipcc, in-tree."""
import glob
import os
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libdynadiag.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-shared",
    "-Wall",
    "-Wno-unused-command-line-argument",
    # packed fp32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build_library(verbose=False):
    """Compile every csrc/*.hip into one shared library.  Always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-o", LIB_PATH, *sources()]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB_PATH


CEILINGS_SRC = os.path.join(PKG_DIR, "ceilings", "ceilings.hip")
CEILINGS_BIN = os.path.join(PKG_DIR, "ceilings", "ceilings")


def build_ceilings():
    """Compile the stand-alone ceilings microbenchmark (not part of the library)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17",
                           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                           "-o", CEILINGS_BIN, CEILINGS_SRC])
    return CEILINGS_BIN


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_ceilings())
