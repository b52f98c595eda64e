"""Builds libmoe_spac.so (HIP, gfx950 only) next to this file.

Each source is compiled to an object of its own (in parallel; objects live in _build/, which is not
tracked) and the objects are linked into the shared library."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmoe_spac.so")
LIB_TRACE = os.path.join(HERE, "libmoe_spac_trace.so")   # same sources with the timeline stamps compiled in
SOURCES = ["api.hip", "route.hip", "ffn.hip", "stream.hip", "layer.hip", "estimator.hip", "balancer.hip", "cache.hip"]
HEADERS = [os.path.join(CSRC, h) for h in ("moe_internal.h", "route_device.h")] + \
          [os.path.join(ROOT, "include", "moe_spac.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # packed-fp32 instruction selection is switched off for every kernel of this library
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


def _sources():
    return [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]


def _headers():
    return [h for h in HEADERS if os.path.exists(h)]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in [os.path.join(CSRC, s) for s in _sources()] + _headers())


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
    if p.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build_hip(force: bool = True, verbose: bool = False, trace: bool = False, jobs: int = 8) -> str:
    """force: recompile every source; otherwise only the objects older than their source or a header."""
    out_path = LIB_TRACE if trace else LIB
    if not (force or trace or stale()):
        return out_path
    os.makedirs(OBJ_DIR, exist_ok=True)
    extra = ["-DMOE_STREAM_TRACE=1"] if trace else []
    newest_header = max(os.path.getmtime(h) for h in _headers())
    objs, todo = [], []
    for s in _sources():
        src = os.path.join(CSRC, s)
        obj = os.path.join(OBJ_DIR, s.replace(".hip", ".trace.o" if trace else ".o"))
        objs.append(obj)
        if force or not os.path.exists(obj) or os.path.getmtime(obj) < max(os.path.getmtime(src), newest_header):
            todo.append(["hipcc"] + FLAGS + extra + ["-c", src, "-o", obj])
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(todo) or 1))) as ex:
        list(ex.map(lambda c: _run(c, verbose), todo))
    _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", out_path], verbose)
    return out_path


if __name__ == "__main__":
    print(build_hip(force="--incremental" not in sys.argv, verbose=True, trace="--trace" in sys.argv))
