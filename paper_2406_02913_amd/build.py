"""Builds libszo.so (host C++ + HIP kernels for gfx950) in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libszo.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

HIP_SOURCES = ["szo_kernels.hip", "szo_gemm.hip", "szo_smallm.hip"]
HOST_SOURCES = ["szo_host.cpp"]

COMMON = ["-O3", "-fPIC", "-std=c++17", "-I", os.path.join(ROOT, "include"), "-I", CSRC]
# packed fp32 VALU forms are switched off (see the hardware notes this project follows)
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)


def build(verbose=False, extra=()):
    """Compiles every source (in parallel: the translation units are independent) and links the library."""
    from concurrent.futures import ThreadPoolExecutor
    jobs, objs = [], []
    for src in HOST_SOURCES:
        obj = os.path.join(CSRC, src + ".o")
        jobs.append(["g++", "-c", "-ffp-contract=off", "-pthread"] + COMMON + [os.path.join(CSRC, src), "-o", obj])
        objs.append(obj)
    for src in HIP_SOURCES:
        obj = os.path.join(CSRC, src + ".o")
        jobs.append([HIPCC, "-c"] + COMMON + DEVICE + list(extra) + [os.path.join(CSRC, src), "-o", obj])
        objs.append(obj)
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as pool:
        list(pool.map(lambda c: _run(c, verbose), jobs))
    _run([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs + ["-lpthread"], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
