"""Builds libmsgemm.so (HIP, gfx950) in-tree with hipcc.  Run as
``python -m paper_2310_06178_amd.build``; ``__graft_entry__.build()`` calls it."""
from __future__ import annotations

import glob
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmsgemm.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = True, defines=(), out: str = LIB) -> str:
    """Compile the library.  `defines` / `out` make a measurement build beside the product (for instance
    MSGEMM_WIDE_LEAVE_OUT=1, see csrc/kernels_fused.hip; bench.py --lib times such a build)."""
    cmd = [hipcc(), *HIPCC_FLAGS, *[f"-D{d}" for d in defines], "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-o", out, *sources()]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("--define", "-D", action="append", default=[], help="preprocessor definition NAME or NAME=VALUE")
    ap.add_argument("--out", default=LIB, help="output path (default: the product library)")
    args = ap.parse_args()
    build(defines=args.define, out=args.out)
    sys.exit(0)
