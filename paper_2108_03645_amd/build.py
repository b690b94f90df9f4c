"""Builds libones.so (HIP, gfx950 only) in-tree next to its sources."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libones.so")
# (source, object, extra flags); the evolve kernel is built once per group of eight row counts
UNITS = [("ones_api.hip", "ones_api.o", []), ("ones_select.hip", "ones_select.o", []),
         ("ones_sample.hip", "ones_sample.o", []), ("ones_fused.hip", "ones_fused.o", [])] + [
    ("ones_evolve.hip", f"ones_evolve_{g}.o", [f"-DONES_ROW_GROUP={g}"]) for g in range(4)]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument", f"-I{INCLUDE}", f"-I{CSRC}",
         *os.environ.get("ONES_EXTRA_FLAGS", "").split()]


HEADERS = [os.path.join(CSRC, h) for h in ("ones_device.h", "ones_sample.h", "ones_candidate.h", "ones_sort.h")] + [
           os.path.join(INCLUDE, "ones.h"),
           os.path.abspath(__file__)]


def _compile(unit, force: bool = True) -> str:
    src, obj, extra = unit
    obj, src = os.path.join(CSRC, obj), os.path.join(CSRC, src)
    fresh = os.path.exists(obj) and all(os.path.getmtime(f) <= os.path.getmtime(obj) for f in [src, *HEADERS])
    if force or not fresh:
        subprocess.check_call([HIPCC, *FLAGS, *extra, "-c", src, "-o", obj])
    return obj


def build(verbose: bool = True, force: bool = True) -> str:
    """Compile every source (force=False: only those older than their inputs) and link the
    shared library; returns its path."""
    with ThreadPoolExecutor(max_workers=min(8, len(UNITS))) as ex:
        objs = list(ex.map(lambda u: _compile(u, force), UNITS))
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB])
    if verbose:
        print(f"built {LIB}", file=sys.stderr)
    return LIB


if __name__ == "__main__":
    build(force="--changed" not in sys.argv)
