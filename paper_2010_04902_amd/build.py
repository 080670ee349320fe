"""Builds libbyzshield.so (HIP kernels + host library + C-ABI) for gfx950, in-tree."""
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libbyzshield.so")
SOURCES = [os.path.join(CSRC, "kernels.hip"), os.path.join(CSRC, "krum.hip"),
           os.path.join(CSRC, "host.cpp")]


def build(verbose=False):
    """Always compiles (seconds to a few minutes); raises on failure."""
    sys.path.insert(0, CSRC)
    try:
        import gen_selnet
        gen_selnet.main(os.path.join(CSRC, "generated"))
    finally:
        sys.path.remove(CSRC)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-Wno-unused-parameter",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC] + SOURCES + ["-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
