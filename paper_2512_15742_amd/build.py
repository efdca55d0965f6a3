"""Builds libkan_mi355x.so (gfx950) in-tree with hipcc.

    python -m paper_2512_15742_amd.build

Objects go to `_build/` at the repository root (not committed); the shared
library lands next to this file so that it travels with the source tree.
hipcc cross-compiles for gfx950 without a GPU being present.
"""
from __future__ import annotations

import concurrent.futures as cf
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(ROOT, "_build")
LIB = os.path.join(HERE, "libkan_mi355x.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

COMMON = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # packed fp32 VALU forms are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]

# (source, object name, extra flags)
UNITS = [
    ("kan_api.hip", "kan_api.o", []),
    ("kan_misc.hip", "kan_misc.o", []),
    ("kan_mfma.hip", "kan_mfma.o", []),
    ("kan_fused.hip", "kan_fused.o", []),
    ("kan_fused.hip", "kan_fused_chained.o", ["-DKAN_FUSED_CH=1"]),
    ("kan_bucket.hip", "kan_bucket.o", []),
    ("kan_assign.hip", "kan_assign.o", []),
    ("kan_gather.hip", "kan_gather_bt1.o", ["-DKAN_BT=1"]),
    ("kan_gather.hip", "kan_gather_bt4.o", ["-DKAN_BT=4"]),
    ("kan_gather.hip", "kan_gather_bt16.o", ["-DKAN_BT=16"]),
]


def _compile(unit, extra_flags):
    src, obj, flags = unit
    cmd = [HIPCC, *COMMON, *flags, *extra_flags, "-c", os.path.join(CSRC, src), "-o", os.path.join(BUILD, obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    return unit, r.returncode, r.stdout + r.stderr


def build(verbose: bool = True, extra_flags=(), jobs: int = 6) -> str:
    os.makedirs(BUILD, exist_ok=True)
    with cf.ThreadPoolExecutor(max_workers=jobs) as ex:
        results = list(ex.map(lambda u: _compile(u, list(extra_flags)), UNITS))
    for unit, rc, out in results:
        noise = "unknown feature" in out or "not a recognized feature" in out
        if rc != 0 or (verbose and out.strip() and not noise):
            sys.stderr.write(f"[{unit[1]}] rc={rc}\n{out}\n")
        if rc != 0:
            raise RuntimeError(f"hipcc failed on {unit[0]} ({unit[1]})")
    objs = [os.path.join(BUILD, u[1]) for u in UNITS]
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build()
