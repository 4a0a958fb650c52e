"""Builds libmosaic.so (HIP, gfx950 only) in-tree with hipcc.  No JIT, no fallback."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libmosaic.so")
SOURCES = ["mosaic_api.hip", "mosaic_compact.hip", "mosaic_logits.hip", "mosaic_unmask.hip", "mosaic_probe.hip", "mosaic_vmm.hip",
           "mosaic_plan.cpp", "mosaic_graph.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 VALU forms are kept off for every HIP translation unit
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def build_library(verbose: bool = False) -> str:
    # the hand-scheduled K-loop of the 4-wave kernel is generated text; regenerate it so it cannot go stale
    subprocess.run([sys.executable, os.path.join(CSRC, "gen_w4_loop.py")], check=True,
                   stdout=None if verbose else subprocess.DEVNULL)
    cmd = [HIPCC, *FLAGS, "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-o", LIB,
           *[os.path.join(CSRC, s) for s in SOURCES]]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    noise = "is not a recognized feature for this target"
    out = "\n".join(l for l in res.stdout.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
