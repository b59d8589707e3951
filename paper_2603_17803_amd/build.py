"""Builds libswarm.so (the HIP library behind include/swarm.h) for gfx950 with hipcc, in-tree."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libswarm.so")
SOURCES = ["api.hip", "score.hip", "select.hip", "coact.hip", "mapper.hip", "density.hip", "window.hip", "retrieval.hip", "calib.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # the fully unrolled epilogues of the co-activation kernel exceed the default budget of "#pragma unroll";
         # a loop left rolled there indexes the accumulator array dynamically and sends it to scratch memory
         "-mllvm", "-pragma-unroll-threshold=200000"]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
