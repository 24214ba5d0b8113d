"""Builds librbe_hip.so (gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librbe_hip.so")
SOURCES = [os.path.join(CSRC, "rbe_api.hip")]
HEADERS = [os.path.join(CSRC, "rbe_kernels.hpp"), os.path.join(CSRC, "rbe_layout.hpp"),
           os.path.join(ROOT, "include", "rbe.h")]


def hipcc_command(out: str = LIB) -> list[str]:
    return [
        os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"),
        "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wall", "-Wno-unused-function",
        "-I", os.path.join(ROOT, "include"), "-I", CSRC,
        "-o", out, *SOURCES,
    ]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile the library.  With force=False, only when missing."""
    if force or not os.path.exists(LIB):
        cmd = hipcc_command()
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build(force=True, verbose=True)
