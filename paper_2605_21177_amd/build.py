"""Builds libchunkft.so (HIP kernels + C ABI) for gfx950, in-tree.

Every source is compiled to its own object (in parallel), then linked.  `python -m
paper_2605_21177_amd.build` and `build_library()` compile everything every time;
`build_library(only_changed=True)` (or `--changed`) re-uses objects that are newer than their
source and every header, for quick edit-compile cycles.
"""

from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libchunkft.so")
LIB_TIMELINE = os.path.join(PKG, "libchunkft_timeline.so")   # diagnostic twin: workgroups note their phase times

SOURCES = ["kernels.hip", "static_ws.hip", "calib.hip", "api.cpp", "shape.cpp", "plan.cpp", "mover.cpp"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                      # fused and un-fused AdamW must round alike
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-x", "hip",
]

_NOISE = "is not a recognized feature for this target"


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if _NOISE not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def _headers():
    hs = [os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include"))]
    hs += [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".h", ".inc"))]
    return hs


def build_library(verbose: bool = False, only_changed: bool = False, timeline: bool = True) -> str:
    """libchunkft.so, and with `timeline` also libchunkft_timeline.so (kernels.hip built once more with
    -DCHUNKFT_TIMELINE; the other objects are shared)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    newest_header = max(os.path.getmtime(h) for h in _headers())
    jobs = []
    objs = []

    def want(src, obj, extra=()):
        fresh = os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header)
        if not (only_changed and fresh):
            jobs.append([hipcc] + FLAGS + list(extra) + ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", src, "-o", obj])

    for s in SOURCES:
        obj = os.path.join(OBJ, os.path.splitext(s)[0] + ".o")
        objs.append(obj)
        want(os.path.join(CSRC, s), obj)
    tl_obj = os.path.join(OBJ, "kernels_timeline.o")
    if timeline:
        want(os.path.join(CSRC, "kernels.hip"), tl_obj, ["-DCHUNKFT_TIMELINE"])
    workers = max(1, min(len(jobs), os.cpu_count() or 1, 16))
    with ThreadPoolExecutor(max_workers=workers) as pool:
        list(pool.map(lambda c: _run(c, verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB], verbose)
    if timeline:
        tl_objs = [tl_obj if o.endswith(os.sep + "kernels.o") else o for o in objs]
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + tl_objs + ["-o", LIB_TIMELINE], verbose)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True, only_changed="--changed" in sys.argv[1:]))
    sys.exit(0)
