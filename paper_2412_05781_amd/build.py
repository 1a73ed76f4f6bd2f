"""Compile libwino.so for gfx950 with hipcc (in-tree, no JIT cache).

Each source is compiled to an object of its own (in parallel), then linked.  `build_libwino()` always
recompiles everything; `--incremental` on the command line reuses objects newer than every source and header.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libwino.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CFLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 code generation is switched off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I" + os.path.join(ROOT, "include"),
]
NOISE = "packed-fp32-ops"       # the host pass does not know the device feature and says so


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _headers():
    return glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if NOISE not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + out)
    return out


def build_libwino(verbose: bool = False, incremental: bool = False, jobs: int = 8) -> str:
    """Returns the path of the shared library."""
    os.makedirs(OBJ, exist_ok=True)
    newest_header = max(os.path.getmtime(h) for h in _headers())
    todo, objs = [], []
    for src in sources():
        obj = os.path.join(OBJ, os.path.basename(src)[:-4] + ".o")
        objs.append(obj)
        fresh = os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header)
        if not (incremental and fresh):
            todo.append([HIPCC] + CFLAGS + ["-c", src, "-o", obj])
    if verbose:
        for cmd in todo:
            print(" ".join(cmd), flush=True)
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(todo) or 1))) as pool:
        outs = list(pool.map(_run, todo))
    link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-Wno-unused-command-line-argument"] + objs + ["-o", LIB]
    if verbose:
        print(" ".join(link), flush=True)
    outs.append(_run(link))
    if verbose:
        text = "\n".join(o for o in outs if o.strip())
        if text:
            print(text)
    return LIB


if __name__ == "__main__":
    print(build_libwino(verbose=True, incremental="--incremental" in sys.argv))
