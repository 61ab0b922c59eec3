"""Builds libpsgd.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libpsgd.so")
SOURCES = ["psgd_plan.cpp", "psgd_kernels.hip", "psgd_resident.hip", "psgd_highrank.hip", "psgd_sparse.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "-shared",
    "--offload-arch=gfx950",
    # no packed-FP32 instructions from the auto-vectoriser
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fvisibility=hidden", "-Wall", "-Wno-unused-function",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    return res.stdout


def build_library(verbose: bool = False) -> str:
    """Compile every source for gfx950 (one hipcc process per source, side by side) and link libpsgd.so next to
    this file.  The objects live in a temporary folder outside the tree."""
    compile_flags = [f for f in FLAGS if f != "-shared"]
    tmp = tempfile.mkdtemp(prefix="psgd_build_")
    try:
        objs = [os.path.join(tmp, os.path.splitext(s)[0] + ".o") for s in SOURCES]
        cmds = [[HIPCC] + compile_flags + ["-c", "-x", "hip", os.path.join(CSRC, s), "-o", o]
                for s, o in zip(SOURCES, objs)]
        with concurrent.futures.ThreadPoolExecutor(max_workers=min(len(cmds), os.cpu_count() or 1)) as pool:
            outs = list(pool.map(lambda c: _run(c, verbose), cmds))
        outs.append(_run([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950"] + objs + ["-o", LIB_PATH], verbose))
        if verbose:
            for o in outs:
                if o.strip():
                    print(o)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return LIB_PATH


if __name__ == "__main__":
    build_library(verbose=True)
    print("built", LIB_PATH)
    sys.exit(0)
