"""Compile csrc/ into libmpcnn.so for gfx950 with hipcc (cross-compiles without a GPU).

    python -m paper_1302_1690_amd.build

Every .hip file under csrc/ is one translation unit (the host side, and one per family of
matrix-core kernel instances); they are compiled side by side and linked into one library.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmpcnn.so")
OBJ = os.path.join(HERE, "_build")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed fp32 arithmetic
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def build_lib(verbose: bool = True, only=None) -> str:
    """Compile every translation unit (or, with `only`, those whose file name contains one of
    the given strings, reusing the other objects of an earlier build) and link the library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    inc = ["-I", os.path.join(HERE, "..", "include")]
    jobs = []
    for s in sources():
        o = os.path.join(OBJ, os.path.basename(s)[:-4] + ".o")
        if only and not any(t in os.path.basename(s) for t in only) and os.path.exists(o):
            jobs.append((None, o))
            continue
        jobs.append(([hipcc] + HIPCC_FLAGS + inc + ["-c", s, "-o", o], o))

    def run(job):
        cmd, _ = job
        if cmd is None:
            return
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)

    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        list(ex.map(run, jobs))
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + [o for _, o in jobs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    build_lib(only=sys.argv[1:] or None)
    sys.exit(0)
