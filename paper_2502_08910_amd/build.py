"""Builds libihip.so (gfx950) in-tree with hipcc.  `python -m paper_2502_08910_amd.build`.

Every source is compiled to an object of its own (in parallel, under
paper_2502_08910_amd/_build/) and the objects are linked into the library."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libihip.so")
SOURCES = ["api.hip", "prune_stage.hip", "prune_prefill_fp8.hip", "prune_stage_rope.hip", "select_blocks.hip", "sparse_attn_decode.hip",
           "sparse_attn_prefill.hip", "sparse_attn_prefill32.hip", "sparse_attn_prefill32_fp8.hip", "cache.hip", "mfma_rate.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option"]
# The pruning kernels take maxima of matrix-core results; told that NaNs need not be honoured the
# compiler drops the canonicalising v_max x,x,x in front of each (a third of the vector
# instructions of the prefill search loop).  Scores of NaN inputs are then unspecified values.
EXTRA = {"prune_stage.hip": ["-fno-honor-nans"], "prune_prefill_fp8.hip": ["-fno-honor-nans"]}


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJ, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *EXTRA.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        return obj

    with ThreadPoolExecutor(max_workers=min(os.cpu_count() or 8, len(SOURCES))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
