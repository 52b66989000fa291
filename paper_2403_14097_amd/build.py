"""Builds the HIP library for gfx950 in-tree: python -m paper_2403_14097_amd.build"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "parcae_api.hip")
LIB = os.path.join(HERE, "libparcae_hip.so")

FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fPIC", "-shared", "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def build(verbose: bool = False, extra: list[str] | None = None) -> str:
    """Compile the library with hipcc (always recompiles)."""
    cmd = ["hipcc", *FLAGS, *(extra or []), "-o", LIB, SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
