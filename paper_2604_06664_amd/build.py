"""Builds libfdy.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2604_06664_amd.build`"""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libfdy.so")
SOURCES = ["fdy_api.hip", "fdy_scan.hip", "fdy_fingerprint.hip", "fdy_materialize.hip", "fdy_derive.hip",
           "fdy_arena.hip", "fdy_archive.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra",
    "-Wno-unused-parameter",
    # packed-fp32 instruction forms stay disabled for all device code in this repository
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def hipcc():
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def build_lib(verbose=False):
    cmd = [hipcc()] + FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    cmd += [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


TOY_SRC = [os.path.join(ROOT, "tests", "toy_graph", f) for f in ("toy_graph.hip", "install_scale.hip",
                                                                "arena_graph.hip")]
TOY_LIB = os.path.join(ROOT, "tests", "toy_graph", "libtoy_graph.so")


def build_toy(verbose=False):
    """The toy hipGraph end-to-end checks (test programs; link against libfdy.so)."""
    cmd = [hipcc()] + FLAGS + ["-I", os.path.join(ROOT, "include")] + TOY_SRC + ["-L", PKG, "-lfdy",
                               "-Wl,-rpath,$ORIGIN/../../paper_2604_06664_amd", "-o", TOY_LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return TOY_LIB


if __name__ == "__main__":
    build_lib(verbose=True)
    print("built", LIB)
    build_toy(verbose=True)
    print("built", TOY_LIB)
    sys.exit(0)
