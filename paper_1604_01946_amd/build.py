"""Builds the HIP library in-tree for gfx950 (hipcc cross-compiles without a GPU): every translation unit is
compiled on its own, a few at a time, and the objects are linked into one shared library."""
import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG_DIR, "liblstm_mi355x.so")
OBJ_DIR = os.path.join(PKG_DIR, "_build")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "is not a recognized feature for this target" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build_library(verbose=False, jobs=None):
    srcs = sorted(glob.glob(os.path.join(PKG_DIR, "csrc", "*.hip")))
    os.makedirs(OBJ_DIR, exist_ok=True)
    objs = [os.path.join(OBJ_DIR, os.path.basename(s)[:-4] + ".o") for s in srcs]
    jobs = jobs or min(8, int(os.environ.get("MAX_JOBS", "8")), len(srcs))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        list(pool.map(lambda so: _run([HIPCC] + FLAGS + ["-c", so[0], "-o", so[1]], verbose), zip(srcs, objs)))
    _run([HIPCC, "--offload-arch=gfx950", "-fPIC", "-shared"] + objs + ["-o", LIB_PATH], verbose)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
