"""Builds librbe_hip.so (gfx950) in-tree with hipcc.

The scan kernel families are compiled once per word count (dim / 64) as separate
objects, in parallel, and linked with the host code into one shared library.
"""
from __future__ import annotations

import os
import subprocess
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librbe_hip.so")
HEADERS = [os.path.join(CSRC, h) for h in ("rbe_kernels.hpp", "rbe_layout.hpp", "rbe_internal.hpp",
                                           "rbe_misc_kernels.hpp")] + [os.path.join(ROOT, "include", "rbe.h"), os.path.join(ROOT, "include", "rbe_debug.h")]
# (source, extra defines, object suffix)
# The matrix-core kernel reads every accumulator with ordinary vector instructions right after the MFMAs:
# keep the accumulators in the ordinary register file (gfx950 has one unified file) instead of copying
# each result out of the accumulation registers first.
MFMA_VGPR = ["-mllvm", "-amdgpu-mfma-vgpr-form"]
UNITS = [("rbe_api.hip", [], "api")] + \
        [("rbe_scan.hip", [f"-DRBE_W={w}"], f"scan_w{w}") for w in (1, 2, 4)] + \
        [("rbe_group.hip", [f"-DRBE_W={w}"], f"group_w{w}") for w in (1, 2, 4)] + \
        [("rbe_batch.hip", [f"-DRBE_W={w}", *MFMA_VGPR], f"batch_w{w}") for w in (1, 2)]
SOURCES = sorted({os.path.join(CSRC, u[0]) for u in UNITS})

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wall", "-Wno-unused-function", "-Wno-unused-command-line-argument",
          "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False, out: str = LIB, extra_flags=()) -> str:
    """Compile the library.  With force=False, only when missing."""
    if not force and os.path.exists(out):
        return out
    with tempfile.TemporaryDirectory(prefix="rbe_build_") as tmp:
        procs, objs = [], []
        for src, defs, tag in UNITS:
            obj = os.path.join(tmp, tag + ".o")
            cmd = [HIPCC, *COMMON, *extra_flags, *defs, "-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
            objs.append(obj)
        failed = []
        for cmd, pr in procs:
            log, _ = pr.communicate()
            log = "\n".join(l for l in log.splitlines() if "packed-fp32-ops" not in l)
            if pr.returncode != 0:
                failed.append((cmd, log))
            elif verbose and log.strip():
                print(log, flush=True)
        if failed:
            raise RuntimeError("hipcc failed:\n" + "\n".join(" ".join(c) + "\n" + o for c, o in failed))
        link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.check_call(link)
    return out


if __name__ == "__main__":
    build(force=True, verbose=True)
