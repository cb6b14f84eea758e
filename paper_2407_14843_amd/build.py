"""Compile the HIP sources into shared libraries (gfx950 only).

    csrc/*.hip            -> libthemis_hip.so    the solve, behind include/themis.h
    probe/lds_probe.hip   -> libthemis_probe.so  LDS / vector-issue probes that only
                                                 the benchmark loads

hipcc cross-compiles without a GPU.  The libraries are built in-tree, next to
this file, so that they travel with the source tree.
"""

from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB_PATH = os.path.join(HERE, "libthemis_hip.so")
PROBE_LIB_PATH = os.path.join(HERE, "libthemis_probe.so")
SOURCES = ["themis_api.hip", "k1_candidates.hip", "k2_minplus.hip", "k2_steps.hip",
           "k3_backtrack.hip",
           "k4_fallback.hip", "k5_stability.hip", "k6_memo.hip"]
PROBE_SOURCES = [os.path.join(HERE, "probe", "lds_probe.hip")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def build(verbose: bool = False, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    base = [hipcc] + HIPCC_FLAGS + list(extra_flags) + ["-I", INCLUDE, "-I", CSRC]
    for sources, out in (([os.path.join(CSRC, s) for s in SOURCES], LIB_PATH),
                         (PROBE_SOURCES, PROBE_LIB_PATH)):
        cmd = base + sources + ["-o", out]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
    return LIB_PATH


if __name__ == "__main__":
    build(verbose=True, extra_flags=sys.argv[1:])
