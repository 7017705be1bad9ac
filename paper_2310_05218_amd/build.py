"""Builds libswconv.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libswconv.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    # packed-FP32 VALU forms are switched off for every kernel in this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = False, jobs: int = 8) -> str:
    """Compile every kernel and the C ABI into ``libswconv.so``; always recompiles.  The translation units
    are compiled side by side into ``_build/`` at the repository root (not tracked), then linked."""
    import concurrent.futures
    import shutil

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    inc = ["-I", os.path.join(PKG, "..", "include")]
    tmp = os.path.join(PKG, "..", "_build")
    shutil.rmtree(tmp, ignore_errors=True)
    os.makedirs(tmp)
    try:
        # the source of the run-time-compiled kernel travels inside the library as a string literal
        with open(os.path.join(CSRC, "jit", "sliding_plane_jit.hip")) as f:
            text = f.read()
        assert ')SWJIT"' not in text
        with open(os.path.join(tmp, "sw_jit_source.inc"), "w") as f:
            f.write('R"SWJIT(' + text + ')SWJIT"\n')
        inc += ["-I", tmp]

        def compile_one(src):
            obj = os.path.join(tmp, os.path.basename(src) + ".o")
            cmd = [hipcc, *HIPCC_FLAGS, *inc, "-c", src, "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True)
            return obj

        with concurrent.futures.ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
            objs = list(pool.map(compile_one, sources()))
        cmd = [hipcc, "--offload-arch=gfx950", "-fPIC", "-shared", "-o", LIB, *objs, "-lhiprtc"]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
