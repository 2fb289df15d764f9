"""Compile the HIP library for gfx950 into paper_2601_16991_amd/libsalr_hip.so (in-tree).

Every source is compiled to an object of its own (in parallel), then linked; `python build.py --changed` skips
objects that are newer than their source and every header (for quick rebuilds while working on one kernel)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsalr_hip.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    # packed-fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall",
    "-Wno-unused-function",
    # the LDS-DMA loads are issued from inline assembly that sets m0 and says so in its clobber list; the compiler
    # remarks on every such statement that m0 is a reserved register
    "-Wno-inline-asm",
]


def sources() -> list[str]:
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _headers() -> list[str]:
    return sorted(glob.glob(os.path.join(CSRC, "*.hpp")) + glob.glob(os.path.join(ROOT, "include", "*.h")))


def _run(cmd: list[str]) -> str:
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + out)
    return out


def build(verbose: bool = False, only_changed: bool = False, jobs: int | None = None) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    newest_header = max(os.path.getmtime(h) for h in _headers())
    todo, objects = [], []
    for src in sources():
        obj = os.path.join(OBJ_DIR, os.path.basename(src)[:-4] + ".o")
        objects.append(obj)
        fresh = os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header)
        if not (only_changed and fresh):
            todo.append([hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", "-o", obj, src])
    if jobs is None:
        jobs = min(8, max(1, len(os.sched_getaffinity(0))))
    if verbose:
        for cmd in todo:
            print(" ".join(cmd), flush=True)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        outs = list(pool.map(_run, todo))
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objects]
    if verbose:
        print(" ".join(link), flush=True)
    outs.append(_run(link))
    text = "\n".join(o for o in outs if o.strip())
    if verbose and text:
        print(text)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, only_changed="--changed" in sys.argv[1:]))
    sys.exit(0)
