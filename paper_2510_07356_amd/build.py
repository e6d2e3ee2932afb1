"""Build libgqa_decode.so for gfx950 with hipcc (in-tree, next to this file)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgqa_decode.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 VALU forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build_library(verbose: bool = False, out: str = LIB, defines=()) -> str:
    """defines: extra -D tunables (see the #ifndef blocks at the top of the kernels)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *[f"-D{d}" for d in defines], "-o", out, *sources()]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout)
        raise RuntimeError("hipcc failed")
    if verbose and res.stdout.strip():
        print(res.stdout)
    return out


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser(description="build libgqa_decode.so (default: in-tree, default tunables)")
    ap.add_argument("--out", default=LIB, help="output path; load it with GQA_DECODE_LIBRARY=<path>")
    ap.add_argument("-D", dest="defines", action="append", default=[],
                    help="compile-time tunable, e.g. -D GQA_MFMA_WGS_PER_CU=2 (see the #ifndef blocks in csrc/)")
    a = ap.parse_args()
    print(build_library(verbose=True, out=a.out, defines=a.defines))
