"""The library's host code (argument validation, dispatch, the static-scratch bookkeeping) built with
AddressSanitizer and UndefinedBehaviorSanitizer and driven through every entry point's error paths on the
CPU.  Sanitizers run on host code only: nothing here touches a GPU, and no GPU run is ever sanitized.
(The oracle is numpy code; there is no native oracle code to put under a sanitizer.)"""
import os
import shutil
import subprocess

import pytest

from paper_2605_14292_amd import build as BLD

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="no hipcc")
def test_host_code_under_asan_and_ubsan(tmp_path):
    objs = [os.path.join(BLD.OBJ, s.replace(".hip", ".o")) for s in BLD.SOURCES]
    if not all(os.path.exists(o) for o in objs):
        BLD.build(verbose=False, only_changed=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    api_o = str(tmp_path / "kvr_api_san.o")
    drv_o = str(tmp_path / "host_abi_checks.o")
    exe = str(tmp_path / "host_abi_checks")
    subprocess.run([HIPCC] + BLD.FLAGS + san + ["-g", "-c", os.path.join(BLD.CSRC, "kvr_api.hip"), "-o", api_o],
                   check=True, stderr=subprocess.DEVNULL)
    subprocess.run(["/opt/rocm/lib/llvm/bin/clang" if os.path.exists("/opt/rocm/lib/llvm/bin/clang") else "clang",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-g", "-c",
                    os.path.join(ROOT, "tests", "host_abi_checks.c"), "-o", drv_o], check=True)
    others = [o for o in objs if not o.endswith("kvr_api.o")]
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize"] + others + [api_o, drv_o, "-o", exe],
                   check=True, stderr=subprocess.DEVNULL)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "host checks ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
