"""Builds libkvr.so (the HIP kernels and the C-ABI) for gfx950 with hipcc,
in-tree next to the sources, and libkvr_bounds.so, the same sources with the
bounds checks of csrc/kvr_bounds.hpp compiled in (-DKVR_BOUNDS; a debug aid that
the GPU tests run beside the product library).  Every source is compiled to an
object of its own (in parallel), then linked; `python -m paper_2605_14292_amd.build
--changed` recompiles only the sources that are newer than their objects."""
from __future__ import annotations

import concurrent.futures
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libkvr.so")
OBJ_BOUNDS = os.path.join(HERE, "_build_bounds")
LIB_BOUNDS = os.path.join(HERE, "libkvr_bounds.so")
SOURCES = ["kvr_api.hip", "kvr_score.hip", "kvr_score_wide.hip", "kvr_select_generic.hip", "kvr_compact.hip",
           "kvr_retain_dense.hip", "kvr_retain_dense16.hip", "kvr_select_dense_f32.hip", "kvr_signature_flat.hip",
           "kvr_score_prior.hip", "kvr_score_pool.hip", "kvr_budget.hip", "kvr_retain_pruned.hip",
           "kvr_select_pool.hip", "kvr_select_lazy.hip", "kvr_retain_sparse.hip", "kvr_select_topb.hip", "kvr_validate.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _stale(src: str, obj: str) -> bool:
    if not os.path.exists(obj):
        return True
    t = os.path.getmtime(obj)
    deps = [src] + glob.glob(os.path.join(CSRC, "*.hpp")) + glob.glob(os.path.join(HERE, "..", "include", "*.h"))
    return any(os.path.getmtime(d) > t for d in deps)


def build(verbose: bool = True, only_changed: bool = False, extra_flags=()) -> str:
    """Both libraries: the product, then the one with bounds checks."""
    lib = _build_one(OBJ, LIB, verbose, only_changed, tuple(extra_flags))
    _build_one(OBJ_BOUNDS, LIB_BOUNDS, verbose, only_changed, tuple(extra_flags) + ("-DKVR_BOUNDS",))
    return lib


def _build_one(obj_dir: str, lib_path: str, verbose: bool, only_changed: bool, extra_flags) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(obj_dir, exist_ok=True)
    jobs = []
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(obj_dir, s.replace(".hip", ".o"))
        if only_changed and not _stale(src, obj):
            continue
        jobs.append([hipcc] + FLAGS + list(extra_flags) + ["-c", src, "-o", obj])

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True, stderr=subprocess.DEVNULL if not verbose else None)

    workers = max(1, min(8, os.cpu_count() or 1))
    with concurrent.futures.ThreadPoolExecutor(workers) as pool:
        list(pool.map(run, jobs))
    objs = [os.path.join(obj_dir, s.replace(".hip", ".o")) for s in SOURCES]
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", lib_path]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    return lib_path


if __name__ == "__main__":
    build(only_changed="--changed" in sys.argv[1:])
    sys.exit(0)
