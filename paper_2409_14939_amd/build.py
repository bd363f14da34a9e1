"""Compile libfastgl_agg.so for gfx950 with hipcc (in-tree, next to this file)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libfastgl_agg.so")
SOURCES = ["api.hip", "bookkeeping.hip", "aggregate.hip", "update.hip", "idmap.hip", "match.hip", "edge.hip",
           "static_scratch.hip", "layer.hip"]


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           # packed-fp32 instruction selection is switched off for all device code
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(HERE, "csrc")]
    cmd += [os.path.join(HERE, "csrc", s) for s in SOURCES]
    cmd += ["-o", LIB]
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
