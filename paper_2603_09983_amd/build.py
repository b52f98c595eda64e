"""Builds libmoe_spac.so (HIP, gfx950 only) next to this file."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmoe_spac.so")
LIB_TRACE = os.path.join(HERE, "libmoe_spac_trace.so")   # same sources with the timeline stamps compiled in
SOURCES = ["api.hip", "route.hip", "ffn.hip", "stream.hip", "estimator.hip", "balancer.hip", "cache.hip"]
HEADERS = [os.path.join(CSRC, "moe_internal.h"), os.path.join(CSRC, "route_device.h"),
           os.path.join(ROOT, "include", "moe_spac.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         # packed-fp32 instruction selection is switched off for every kernel of this library
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in [os.path.join(CSRC, s) for s in SOURCES] + HEADERS)


def build_hip(force: bool = True, verbose: bool = False, trace: bool = False) -> str:
    out_path = LIB_TRACE if trace else LIB
    if force or trace or stale():
        cmd = ["hipcc"] + FLAGS + (["-DMOE_STREAM_TRACE"] if trace else []) + \
              [os.path.join(CSRC, s) for s in SOURCES] + ["-o", out_path]
        if verbose:
            print(" ".join(cmd))
        p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + out)
        if verbose and out.strip():
            print(out)
    return out_path


if __name__ == "__main__":
    print(build_hip(force=True, verbose=True, trace="--trace" in sys.argv))
