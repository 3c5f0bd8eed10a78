"""Compile the HIP sources into paper_1609_07228_amd/libefanna_hip.so (gfx950)."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = [os.path.join(_HERE, "csrc", f) for f in ("trees.hip", "graph.hip", "search.hip")]
HEADERS = [os.path.join(_HERE, "csrc", "common.h"),
           os.path.join(os.path.dirname(_HERE), "include", "efanna.h")]
LIB = os.path.join(_HERE, "libefanna_hip.so")


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False) -> str:
    """hipcc for gfx950.  Packed-fp32 instruction selection is switched off on purpose
    (those forms have given wrong results on the target machines)."""
    if not force and not stale():
        return LIB
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-o", LIB] + SOURCES
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout, res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
