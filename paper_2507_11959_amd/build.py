"""Build step of the potq HIP library: hipcc, gfx950 only, in-tree shared object."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(_HERE), "include")
LIB_PATH = os.path.join(_HERE, "libpotq.so")
OBJ_DIR = os.path.join(_HERE, "_build")
SOURCES = ["api.hip", "dequant.hip", "repack.hip", "gemv.hip", "gemv_exp.hip", "gemv_canonical.hip", "gemm.hip", "quantize.hip", "fakequant.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = False, jobs: int | None = None) -> str:
    """Compile every kernel source and link paper_2507_11959_amd/libpotq.so (always recompiles).

    The sources are independent translation units (no relocatable device code), so they are
    compiled side by side, one hipcc process each, and linked once.
    """
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    if jobs is None:
        jobs = max(1, min(len(SOURCES), len(os.sched_getaffinity(0)), 16))

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc, *HIPCC_FLAGS, "-I", INCLUDE, "-I", CSRC, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objects = list(pool.map(compile_one, SOURCES))
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objects, "-o", LIB_PATH]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.check_call(link)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
