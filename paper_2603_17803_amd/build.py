"""Builds libswarm.so (the HIP library behind include/swarm.h) for gfx950 with hipcc, in-tree.

Every source is compiled on its own (in parallel) and the objects are linked into one shared library.  A hash
of the sources, the header and the flags is compiled in (swarm_source_hash), so that a library left behind by
an older tree can be told from a current one.
"""
import concurrent.futures
import hashlib
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libswarm.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["api.hip", "score.hip", "select.hip", "coact.hip", "mapper.hip", "density.hip", "window.hip", "retrieval.hip",
           "calib.hip", "noalloc.hip"]
HEADERS = ["common.h", "wave_ops.h", "select_core.h"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # the fully unrolled epilogues of the co-activation kernel exceed the default budget of "#pragma unroll";
         # a loop left rolled there indexes the accumulator array dynamically and sends it to scratch memory
         "-mllvm", "-pragma-unroll-threshold=200000"]


def source_hash() -> str:
    """sha256 over the library's sources, headers and compiler flags, in a fixed order."""
    h = hashlib.sha256()
    files = [os.path.join(CSRC, f) for f in SOURCES + HEADERS] + [os.path.join(ROOT, "include", "swarm.h")]
    for path in files:
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    h.update(" ".join(FLAGS).encode())
    return h.hexdigest()[:32]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    common = [hipcc, *FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, f'-DSWARM_SOURCE_HASH="{source_hash()}"']

    def compile_one(src):
        obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        cmd = [*common, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return obj

    jobs = min(len(SOURCES), int(os.environ.get("MAX_JOBS", os.cpu_count() or 4)), 16)
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
