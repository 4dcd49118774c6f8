"""Builds libsensei_hip.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB_PATH = os.path.join(HERE, "libsensei_hip.so")
SOURCES = ["sparse_kernels.hip", "gemm_kernels.hip", "api.hip"]


def build(verbose: bool = False) -> str:
    """Compiles every HIP source for gfx950 (hipcc cross-compiles without a GPU)."""
    srcs = [os.path.join(HERE, "csrc", s) for s in SOURCES]
    cmd = ["hipcc", "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared", "-Wno-unused-command-line-argument",
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(HERE, "csrc"),
           # packed fp32 instructions are kept out of the generated code
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           *srcs, "-o", LIB_PATH]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libsensei_hip.so")
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
