"""Builds libmoe_gfx950.so (the C-ABI library of include/moe.h) in-tree with hipcc.

usage: python -m paper_2603_06350_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libmoe_gfx950.so")
SOURCES = ["route.hip", "dispatch.hip", "ffn.hip", "combine.hip", "scaler.hip", "status.hip"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def build(verbose: bool = False, extra=(), out: str = LIB) -> str:
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, *extra,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return out


MICROBENCH = ["mfma_rate", "l2_to_lds_stream", "hbm_read_stream"]


def build_microbench(verbose: bool = False) -> list:
    """The stand-alone micro-benchmarks under csrc/microbench (context for the rooflines)."""
    outs = []
    for name in MICROBENCH:
        src = os.path.join(CSRC, "microbench", name + ".hip")
        out = os.path.join(CSRC, "microbench", name + ".exe")
        cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", src, "-o", out]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + res.stderr)
        outs.append(out)
    return outs


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_microbench(verbose=True))
