"""Build libcomet.so (hipcc, gfx950) next to this file.

Usage: python -m paper_2111_09562_amd.build [--force]
The library is built in-tree so that it travels with the source snapshot to the
GPU machine; nothing is compiled at import time.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcomet.so")
ARCH = "gfx950"

FLAGS = [
    "-O3", "-std=c++17", f"--offload-arch={ARCH}", "-fPIC",
    "-ffp-contract=off", "-fno-fast-math",            # every float op is one IEEE operation, as in the reference
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]
OBJ = os.path.join(HERE, "_build")                   # object files (not tracked)
JOBS = 8


def hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def units():
    """The translation units: every .hip file.  No kernel calls device code of another unit, so
    no relocatable device code is needed; the longest units come first."""
    names = sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))
    names.sort(key=lambda f: (not f.startswith("k_decompress"), not f.startswith("k_quantize_rows")))
    return [os.path.join(CSRC, f) for f in names]


def headers():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")) + \
        [os.path.join(HERE, "..", "include", "comet.h")]


def build(force: bool = False, verbose: bool = False) -> str:
    """Compile what is out of date (everything with force), several units at a time, and link."""
    os.makedirs(OBJ, exist_ok=True)
    newest_header = max(os.path.getmtime(p) for p in headers())
    cc = hipcc()
    todo, objs = [], []
    for src in units():
        obj = os.path.join(OBJ, os.path.basename(src)[:-4] + ".o")
        objs.append(obj)
        if force or not os.path.exists(obj) or os.path.getmtime(obj) < max(os.path.getmtime(src), newest_header):
            todo.append([cc] + FLAGS + ["-c", src, "-o", obj])
    running = []
    def reap(block_until_below):
        while len(running) > block_until_below:
            proc, cmd = running.pop(0)
            if proc.wait() != 0:
                for other, _ in running:
                    other.kill()
                raise subprocess.CalledProcessError(proc.returncode, cmd)
    for cmd in todo:
        if verbose:
            print(" ".join(cmd), flush=True)
        running.append((subprocess.Popen(cmd), cmd))
        reap(JOBS - 1)
    reap(0)
    if todo or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        cmd = [cc, f"--offload-arch={ARCH}", "-shared", "-fPIC", "-o", LIB] + objs
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
