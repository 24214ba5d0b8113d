"""Compiled-code check (test infrastructure): the scan kernels must keep whole waves inside their wave-wide steps.

The survivor queues of the scan kernels use wave-wide operations (ballots, lane broadcasts,
"lane 0 reserves, everybody copies") inside loops.  They are written so that every loop
around such a step has a wave-uniform trip count; the compiler then branches on scalar
conditions.  If a change lets the compiler tie such a loop to per-lane state instead, it emits
a loop that peels lanes off the execution mask (`s_andn2_b64 exec, exec, ...`) and the lanes
of one wave run ballots and flushes at different times: entries get lost without any fault.

This script compiles every scan unit to gfx950 assembly and lists the kernels that contain
such a lane-peeling loop.  Kernels whose loops are per-lane by design (the dense debug dumps,
the table load at the start of the hybrid scan) are expected and named below; anything else
is reported and makes the script exit with status 1.

    python tests/check_isa.py        # takes a few minutes; tests/test_binding_cpu.py runs it
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_1802_06466_amd import _build  # noqa: E402

# kernel name prefixes whose lane-peeling loops are intended, with the number allowed per kernel
EXPECTED = {"dense_scores": 1, "dense_scores_fq": 1, "scan_exact_fq": 1, "scan_exact_fq_prog": 1, "scan_exact_fq_prog_hint": 1,
            "scan_exact_fq_prog2_hint": 1}


def kernel_family(mangled: str) -> str:
    m = re.match(r"_ZN3rbe\d+([A-Za-z_0-9]+?)I", mangled)
    return m.group(1) if m else mangled


def main() -> int:
    bad = []
    with tempfile.TemporaryDirectory(prefix="rbe_isa_") as tmp:
        procs = []
        for src, defs, name in _build.UNITS:
            if src == "rbe_api.hip":
                continue
            out = os.path.join(tmp, name + ".s")
            cmd = [_build.HIPCC, *_build.COMMON, *defs, "-S", "--cuda-device-only", "-o", out, os.path.join(_build.CSRC, src)]
            procs.append((name, out, subprocess.Popen(cmd, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)))
        for name, out, pr in procs:
            if pr.wait() != 0:
                print(f"{name}: hipcc failed", file=sys.stderr)
                return 2
            cur, counts = None, {}
            with open(out) as f:
                for line in f:
                    m = re.match(r"^(_ZN\S+):", line)
                    if m:
                        cur = m.group(1)
                        counts[cur] = 0
                    elif cur and "s_andn2_b64 exec, exec," in line:
                        counts[cur] += 1
            n_flagged = 0
            for k, v in counts.items():
                if v > EXPECTED.get(kernel_family(k), 0):
                    bad.append((name, k, v))
                    n_flagged += 1
            print(f"{name}: {len(counts)} kernels, {n_flagged} with unexpected lane-peeling loops", flush=True)
    for name, k, v in bad:
        print(f"UNEXPECTED {name}: {k} ({v})")
    return 1 if bad else 0


if __name__ == "__main__":
    sys.exit(main())
