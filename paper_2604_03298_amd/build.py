"""Builds libenec.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2604_03298_amd.build`.

libenec_test.so is the same library with ENEC_TEST_HOOKS defined for the host code: there the environment
variable ENEC_SPIN_LIMIT lowers the bound of the scan's waits, which the tests of that bound need.

The host code (csrc/enec_api.hip, csrc/enec_pipeline.hip), the kernels for streams with one tuple per data block
(csrc/enec_per_block.hip) and the 18 kernel tables (csrc/enec_kernels.hip, once per element format, group
length and direction) are compiled side by side into _build/*.o and linked into libenec.so.
"""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libenec.so")
TEST_LIB = os.path.join(HERE, "libenec_test.so")      # the same library with ENEC_TEST_HOOKS (tests of the bounded waits)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
SOURCES = [os.path.join(CSRC, "enec_api.hip"), os.path.join(CSRC, "enec_kernels.hip"),
           os.path.join(CSRC, "enec_per_block.hip"), os.path.join(CSRC, "enec_pipeline.hip")]
HEADERS = [os.path.join(CSRC, "enec_device.hpp"), os.path.join(CSRC, "enec_kernels.hpp"),
           os.path.join(CSRC, "enec_per_block.hpp"),
           os.path.join(ROOT, "include", "enec.h")]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-ffp-contract=off",
         "-fPIC", "-I", os.path.join(ROOT, "include")]


def _units():
    units = [("enec_api.o", [SOURCES[0]]), ("enec_api_test.o", ["-DENEC_TEST_HOOKS", SOURCES[0]]),
             ("enec_per_block.o", [SOURCES[2]]), ("enec_pipeline.o", [SOURCES[3]])]
    for lpg in (2, 1, 4):           # lanes per group: group lengths 16, 8, 32
        for dt in (0, 2, 1):
            for direction in (0, 1):
                units.append((f"enec_kernels_dt{dt}_lpg{lpg}_dir{direction}.o",
                              [f"-DENEC_DT={dt}", f"-DENEC_LPG={lpg}", f"-DENEC_DIR={direction}", SOURCES[1]]))
    return units


def build(verbose: bool = False) -> str:
    """Compiles every HIP source for gfx950 (cross-compiles without a GPU) and returns the path."""
    os.makedirs(OBJ, exist_ok=True)

    def compile_one(unit):
        name, args = unit
        cmd = ["hipcc"] + FLAGS + ["-c", "-o", os.path.join(OBJ, name)] + args
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
        return os.path.join(OBJ, name)

    workers = max(1, min(8, os.cpu_count() or 1))
    with ThreadPoolExecutor(workers) as pool:
        objects = list(pool.map(compile_one, _units()))
    api, api_test = os.path.join(OBJ, "enec_api.o"), os.path.join(OBJ, "enec_api_test.o")
    for lib, skip in ((LIB, api_test), (TEST_LIB, api)):
        cmd = ["hipcc", "--offload-arch=gfx950", "-fPIC", "-shared", "-o", lib] + [o for o in objects if o != skip]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc (link) failed:\n" + res.stdout + res.stderr)
    return LIB


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


if __name__ == "__main__":
    print(build(verbose=True))
