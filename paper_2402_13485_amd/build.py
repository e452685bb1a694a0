"""Build the HIP library for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libpropd.so")
SOURCES = ["tree_mask.hip", "tree_attention.hip", "early_prune.hip", "accept_path.hip",
           "commit_path.hip", "tree_controller.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",  # no packed-fp32 codegen
    "-fvisibility=hidden", "-Wall",
]


def build(verbose: bool = False) -> str:
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    extra = os.environ.get("PROPD_EXTRA_HIPCC_FLAGS", "").split()  # tuning experiments only
    cmd = ["hipcc", *FLAGS, *extra, "-DPROPD_BUILD", "-o", LIB_PATH, *srcs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB_PATH


if __name__ == "__main__":
    build(verbose=True)
    print(LIB_PATH)
