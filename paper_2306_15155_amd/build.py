"""Builds libsensei_hip.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB_PATH = os.path.join(HERE, "libsensei_hip.so")
OBJ_DIR = os.path.join(ROOT, "_build")
SOURCES = ["sparse_kernels.hip", "gemm_kernels.hip", "api.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-Wno-unused-command-line-argument",
         "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(HERE, "csrc"),
         # packed fp32 instructions are kept out of the generated code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _run(cmd, verbose):
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd[-3:]))


def build(verbose: bool = False, incremental: bool = False) -> str:
    """Compiles every HIP source for gfx950 (hipcc cross-compiles without a GPU), one translation unit per thread, and links
    the shared library.  incremental=True recompiles only the sources newer than their object file (for development; headers
    are not tracked)."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = [os.path.join(HERE, "csrc", s) for s in SOURCES if os.path.exists(os.path.join(HERE, "csrc", s))]
    objs = [os.path.join(OBJ_DIR, os.path.basename(s) + ".o") for s in srcs]
    todo = [(s, o) for s, o in zip(srcs, objs)
            if not (incremental and os.path.exists(o) and os.path.getmtime(o) >= os.path.getmtime(s))]
    with ThreadPoolExecutor(max_workers=4) as pool:
        list(pool.map(lambda so: _run(["hipcc", *FLAGS, "-c", so[0], "-o", so[1]], verbose), todo))
    _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH], verbose)
    return LIB_PATH


if __name__ == "__main__":
    import sys
    print(build(verbose="-v" in sys.argv, incremental="-i" in sys.argv))
