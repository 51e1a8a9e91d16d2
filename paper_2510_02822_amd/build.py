"""Builds libflexiq.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libflexiq.so")
NUM_TILE_SHAPES = 15
# (source, object, extra flags): the kernel of every tile shape is a translation unit of its own
UNITS = [("pack.hip", "pack.o", []), ("gemm.hip", "gemm.o", []), ("fp6_gemm.hip", "fp6_gemm.o", []),
         ("smallm.hip", "smallm.o", []), ("stream.hip", "stream.o", []), ("conv3.hip", "conv3.o", [])] + \
        [("mixed_tile.hip", "mixed_tile_%d.o" % i, ["-DFQ_TILE=%d" % i]) for i in range(NUM_TILE_SHAPES)]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def build(verbose: bool = False, extra=()) -> str:
    objs = []
    procs = []
    for src, o, defs in UNITS:
        obj = os.path.join(CSRC, o)
        cmd = ["hipcc", *FLAGS, *defs, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for cmd, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), out))
        if verbose and out.strip():
            print(out)
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
