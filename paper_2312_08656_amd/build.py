"""Builds libmaxk.so for gfx950 with hipcc, in-tree (next to this file)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

HERE = Path(__file__).resolve().parent
CSRC = HERE / "csrc"
LIB = HERE / "libmaxk.so"
SOURCES = ["graph.hip", "topk.hip", "spgemm_fwd.hip", "spgemm_fwd_f32.hip", "spgemm_fwd_bf16.hip", "spgemm_fwd_f16.hip",
           "sspmm_bwd.hip", "sspmm_bwd_f32.hip", "sspmm_bwd_bf16.hip", "sspmm_bwd_f16.hip", "sspmm_bwd_tiled.hip", "spmm.hip"]

# -packed-fp32-ops off: the compiler must not form packed fp32 instructions from float code
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unused-result",
]


def build(verbose: bool = False) -> Path:
    """Compile every translation unit and link the shared library (always rebuilds)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    extra = os.environ.get("MAXK_HIPCC_EXTRA", "").split()  # e.g. -DMAXK_FWD_COPY_PAD=4 for an experiment build
    objdir = HERE / "_build"
    objdir.mkdir(exist_ok=True)

    def compile_one(src: str) -> Path:
        obj = objdir / (src + ".o")
        cmd = [hipcc, *HIPCC_FLAGS, *extra, "-c", str(CSRC / src), "-o", str(obj)]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        return obj

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 4)) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    tmp = LIB.with_suffix(".so.tmp%d" % os.getpid())
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *map(str, objs), "-o", str(tmp)]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
