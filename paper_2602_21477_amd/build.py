"""Compile libpancake.so (HIP, gfx950 only) in-tree.

    python -m paper_2602_21477_amd.build            # every source, from scratch
    python -m paper_2602_21477_amd.build --changed  # only sources newer than their objects

Every translation unit is compiled to an object of its own (in parallel) and the objects
are linked into paper_2602_21477_amd/libpancake.so.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libpancake.so")
SOURCES = ["pk_api.hip", "pk_scan.hip", "pk_scan_rq.hip", "pk_select.hip", "pk_worklist.hip", "pk_index.hip", "pk_gemm.hip",
           "pk_kmeans.hip"]
HEADERS = [os.path.join(CSRC, "pk_internal.h"), os.path.join(CSRC, "pk_worklist_dev.h"),
           os.path.join(CSRC, "pk_select_dev.h"),
           os.path.join(ROOT, "include", "pancake.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _quiet(stderr: str) -> str:
    # the host pass does not know the (device-only) packed-fp32 feature and says so once per file
    return "\n".join(l for l in stderr.splitlines() if "packed-fp32-ops" not in l)


def _compile(src: str, extra: list) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    r = subprocess.run(["hipcc"] + FLAGS + extra + ["-c", os.path.join(CSRC, src), "-o", obj], capture_output=True,
                       text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n" + _quiet(r.stderr))
    return _quiet(r.stderr)


def build(verbose: bool = False, changed_only: bool = False, defines: tuple = ()) -> str:
    """Compiles every source (or, with changed_only, those newer than their object) and links."""
    os.makedirs(OBJ, exist_ok=True)
    extra = [f"-D{d}" for d in defines]
    newest_header = max(os.path.getmtime(h) for h in HEADERS)
    todo = []
    for src in SOURCES:
        obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
        stale = (not os.path.exists(obj) or
                 os.path.getmtime(obj) < max(os.path.getmtime(os.path.join(CSRC, src)), newest_header))
        if stale or not changed_only:
            todo.append(src)
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(todo)))) as ex:
        for msg in ex.map(lambda s: _compile(s, extra), todo):
            if verbose and msg.strip():
                print(msg, file=sys.stderr)
    objs = [os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB], capture_output=True,
                       text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, changed_only="--changed" in sys.argv[1:],
                defines=tuple(a[2:] for a in sys.argv[1:] if a.startswith("-D"))))
