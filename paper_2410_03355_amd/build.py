"""Builds liblantern.so (the C-ABI library of include/lantern.h) for gfx950 with hipcc.

hipcc cross-compiles without a GPU.  The library is built in-tree, next to
this file, so that it travels with the source tree.
"""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "liblantern.so")
SOURCES = ("api.hip", "verify.hip", "greedy.hip", "chain.hip", "sequential.hip", "knn.hip", "random_table.hip", "probe.hip")

HIPCC_FLAGS = (
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # every fp operation is rounded on its own: the fp64 kernels reproduce the
    # written formulas operation by operation
    "-ffp-contract=off",
    # no packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
)


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def build(verbose: bool = False) -> str:
    """Compiles every source to an object (in parallel, in a scratch directory) and links the library."""
    import concurrent.futures
    import tempfile

    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    inc = ["-I", os.path.join(_ROOT, "include"), "-I", CSRC]
    with tempfile.TemporaryDirectory(prefix="lantern_build_") as tmp:
        def compile_one(name: str) -> str:
            obj = os.path.join(tmp, os.path.splitext(name)[0] + ".o")
            cmd = [hipcc_path(), *flags, *inc, "-c", os.path.join(CSRC, name), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True)
            return obj

        with concurrent.futures.ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1, 8)) as pool:
            objs = list(pool.map(compile_one, SOURCES))
        link = [hipcc_path(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.run(link, check=True)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
