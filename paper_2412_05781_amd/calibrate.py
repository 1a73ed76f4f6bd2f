"""The microbenchmarks behind the roofline denominators and the statements about what bounds the kernels: a plain copy
kernel (HBM streaming; also the known-size reference the FETCH_SIZE / WRITE_SIZE counters are scaled by), register-only
MFMA rates, the fill rate of a compute unit from L1 / L2 / beyond with ordinary loads and with direct-to-LDS transfers, and
the step (ii) kernel's operand access pattern as a pure stream.  Plain HIP programs under ``calibration/``; nothing in the
library uses them.

    python -m paper_2412_05781_amd.calibrate --build        # hipcc, works without a GPU
    python -m paper_2412_05781_amd.calibrate --run [name]   # on the GPU machine; prints each program's table
"""
from __future__ import annotations

import argparse
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "calibration")
BIN = os.path.join(SRC, "bin")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-result", "-Wno-unused-command-line-argument"]


def names():
    return sorted(os.path.splitext(os.path.basename(p))[0] for p in glob.glob(os.path.join(SRC, "*.hip")))


def build():
    os.makedirs(BIN, exist_ok=True)
    for n in names():
        res = subprocess.run([HIPCC] + FLAGS + [os.path.join(SRC, n + ".hip"), "-o", os.path.join(BIN, n)],
                             stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed on {n}:\n{res.stdout}")
        print("built", n, flush=True)


def run(which):
    for n in names():
        if which and n not in which:
            continue
        exe = os.path.join(BIN, n)
        if not os.path.exists(exe):
            raise RuntimeError(f"{exe} is missing: run with --build first")
        print(f"== {n}", flush=True)
        subprocess.run([exe], check=True, timeout=300)


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--build", action="store_true")
    ap.add_argument("--run", nargs="*", default=None)
    a = ap.parse_args(argv)
    if a.build:
        build()
    if a.run is not None:
        run(a.run)
    if not a.build and a.run is None:
        ap.print_help()


if __name__ == "__main__":
    sys.exit(main())
