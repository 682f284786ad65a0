"""Builds libkvr.so (the HIP kernels and the C-ABI) for gfx950 with hipcc,
in-tree next to the sources."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkvr.so")
SOURCES = ["kvr_api.hip", "kvr_score.hip", "kvr_score_wide.hip", "kvr_select_generic.hip", "kvr_compact.hip",
           "kvr_retain_dense.hip", "kvr_retain_dense16.hip", "kvr_select_dense_f32.hip", "kvr_signature_flat.hip", "kvr_score_prior.hip", "kvr_score_pool.hip", "kvr_budget.hip", "kvr_retain_pruned.hip", "kvr_select_pool.hip", "kvr_select_topb.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
