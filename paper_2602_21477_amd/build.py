"""Compile libpancake.so and the read-pattern probe (HIP, gfx950 only) in-tree.

    python -m paper_2602_21477_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpancake.so")
PROBE_SRC = os.path.join(HERE, "read_pattern_probe.hip")  # measurement aid: the memory system's rate for the scan's load pattern
PROBE = os.path.join(HERE, "read_pattern_probe.bin")
SOURCES = ["pk_api.hip", "pk_scan.hip", "pk_select.hip", "pk_worklist.hip", "pk_index.hip", "pk_gemm.hip", "pk_kmeans.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def build(verbose: bool = False) -> str:
    cmd = ["hipcc"] + FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the (device-only) packed-fp32 feature and says so once per file
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", PROBE_SRC, "-o", PROBE],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed (read_pattern_probe):\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
