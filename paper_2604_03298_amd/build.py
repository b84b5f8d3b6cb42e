"""Builds libenec.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2604_03298_amd.build`."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libenec.so")
SOURCES = [os.path.join(HERE, "csrc", "enec_api.hip")]
HEADERS = [os.path.join(HERE, "csrc", "enec_device.hpp"), os.path.join(ROOT, "include", "enec.h")]


def build(verbose: bool = False) -> str:
    """Compiles every HIP source for gfx950 (cross-compiles without a GPU) and returns the path."""
    cmd = ["hipcc", "-O3", "-std=c++17", "--offload-arch=gfx950",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-ffp-contract=off",
           "-fPIC", "-shared", "-I", os.path.join(ROOT, "include"), "-o", LIB] + SOURCES
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    return LIB


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


if __name__ == "__main__":
    print(build(verbose=True))
