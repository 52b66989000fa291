"""Builds the HIP library for gfx950 in-tree: python -m paper_2403_14097_amd.build"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "parcae_api.hip")
LIB = os.path.join(HERE, "libparcae_hip.so")
LIB_SANITIZED = os.path.join(HERE, "libparcae_hip_asan.so")

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


def build_host_sanitized(verbose: bool = False) -> str:
    """The same library with its HOST code under AddressSanitizer and UndefinedBehaviorSanitizer (device code is
    compiled as usual): for running the argument checks of the entry points under the sanitizers.  A process that
    loads it needs the compiler's sanitizer runtime preloaded (see host_sanitizer_runtime())."""
    host = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
            "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer",
            "-Xarch_host", "-shared-libsan"]
    cmd = ["hipcc", *FLAGS, *host, "-g", "-o", LIB_SANITIZED, SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB_SANITIZED


def host_sanitizer_runtime() -> str:
    out = subprocess.run(["hipcc", "-print-file-name=libclang_rt.asan-x86_64.so"], check=True, capture_output=True,
                         text=True).stdout.strip()
    if not os.path.isabs(out):   # older drivers print the bare name: look in the compiler's runtime directory
        rt = subprocess.run(["/opt/rocm/llvm/bin/clang", "--print-runtime-dir"], check=True, capture_output=True,
                            text=True).stdout.strip()
        for cand in (os.path.join(rt, "libclang_rt.asan.so"), os.path.join(os.path.dirname(rt), "linux", out)):
            if os.path.exists(cand):
                return cand
    return out


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
