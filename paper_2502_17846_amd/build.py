"""Builds libgrem.so (gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "grem.hip")
SRC_EDGE = os.path.join(HERE, "csrc", "grem_edge_stream.hip")
SRC_BUCKETS = os.path.join(HERE, "csrc", "grem_edge_buckets.hip")
SRC_EXPECTED = os.path.join(HERE, "csrc", "grem_expected_cut.hip")
LIB = os.path.join(HERE, "libgrem.so")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
]


def build_library(verbose: bool = False, extra=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, *extra, "-o", LIB, SRC, SRC_EDGE, SRC_BUCKETS, SRC_EXPECTED]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build_library(verbose=True)
