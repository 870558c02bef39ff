"""Compile libtensile.so (HIP kernels + C ABI) for gfx950, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libtensile.so")
SOURCES = ["tas.hip", "eval.hip", "score.hip", "greedy.hip", "link.hip", "workspace.hip", "step.hip"]


def build_library(verbose: bool = False, extra_flags=()) -> str:
    """Every source is compiled (always: nothing is reused from an earlier build), the translation units side
    by side, then linked into the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-I", os.path.join(ROOT, "include"), "-I", CSRC, *extra_flags]
    with tempfile.TemporaryDirectory(prefix="tensile_build_") as tmp:
        objs = [os.path.join(tmp, s.replace(".hip", ".o")) for s in SOURCES]

        def compile_one(pair):
            src, obj = pair
            cmd = [hipcc, *flags, "-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.check_call(cmd)

        with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1, 8)) as pool:
            list(pool.map(compile_one, zip(SOURCES, objs)))
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.check_call(link)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
    sys.exit(0)
