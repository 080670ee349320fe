"""Builds libbyzshield.so (HIP kernels + host library + C-ABI) for gfx950, in-tree."""
import concurrent.futures
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libbyzshield.so")
KERNELS = os.path.join(CSRC, "kernels.hip")
# kernels.hip is compiled once per part (-DBYZ_PART=n): the single-pass kernels are large and
# build in parallel this way
# the slowest parts first: the pool starts them in this order
KERNEL_PARTS = (18, 17, 16, 8, 10, 9, 11, 7, 13, 2, 4, 12, 6, 14, 15, 5, 3, 1, 0)
OTHER_SOURCES = [os.path.join(CSRC, "krum.hip"), os.path.join(CSRC, "host.cpp")]


def build(verbose=False):
    """Always compiles (about three minutes on 8 cores); raises on failure."""
    sys.path.insert(0, CSRC)
    try:
        import gen_selnet
        gen_selnet.main(os.path.join(CSRC, "generated"))
    finally:
        sys.path.remove(CSRC)
    os.makedirs(OBJ, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-Wall", "-Wextra", "-Wno-unused-parameter", "-Wno-unused-function",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    jobs = []
    for part in KERNEL_PARTS:
        obj = os.path.join(OBJ, "kernels_part%d.o" % part)
        jobs.append(([hipcc] + flags + ["-DBYZ_PART=%d" % part, "-c", KERNELS, "-o", obj], obj))
    for src in OTHER_SOURCES:
        obj = os.path.join(OBJ, os.path.splitext(os.path.basename(src))[0] + ".o")
        jobs.append(([hipcc] + flags + ["-c", src, "-o", obj], obj))

    def run(job):
        cmd, obj = job
        import time
        t0 = time.time()
        subprocess.run(cmd, check=True)
        if verbose:
            print("%6.1f s  %s" % (time.time() - t0, " ".join(cmd[-6:])), flush=True)
        return obj

    workers = min(len(jobs), max(1, len(os.sched_getaffinity(0))), 16)
    with concurrent.futures.ThreadPoolExecutor(max_workers=workers) as pool:
        objects = list(pool.map(run, jobs))
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objects + ["-o", LIB]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
