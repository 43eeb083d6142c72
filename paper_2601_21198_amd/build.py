"""Builds libzipmoe.so (host C++ and gfx950 device code) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
# ZIPMOE_LIBRARY points the binding at another build of the same sources (same ABI)
LIB_PATH = os.environ.get("ZIPMOE_LIBRARY", os.path.join(_HERE, "libzipmoe.so"))
SOURCES = [os.path.join(CSRC, f) for f in ("zipmoe_host.cpp", "zipmoe_plan.cpp", "zipmoe_sched.cpp", "zipmoe_decode.hip", "zipmoe_cache.hip", "zipmoe_staged.hip", "zipmoe_probe.hip", "zipmoe_layer.hip")]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"),
]


def build_library(verbose: bool = False) -> str:
    cmd = [HIPCC, *FLAGS, "-x", "hip", *SOURCES, "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
