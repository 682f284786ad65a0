"""The debug build of the library (libkvr_bounds.so: every index that the kernels for heads of more
than 256 tokens compute from the data goes through a range check that records and clamps) gives the
product library's results bit for bit, and no check fails.  The record itself is shown to work by the
self-test entry point, which checks an out-of-range value without touching memory through it."""
import numpy as np
import pytest
import torch

from paper_2605_14292_amd import binding as B
from paper_2605_14292_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _mk(h, n, seed, dtype, scale):
    g = torch.Generator().manual_seed(seed)
    V = torch.randn((h, n, 128), generator=g)
    V[:, n // 2:] = V[:, : n - n // 2] + 0.05 * V[:, n // 2:]          # near-duplicates: the penalty bites
    K = torch.randn((h, n, 128), generator=g)
    s = torch.randn((h, n), generator=g).exp() * scale
    return K.to(dtype).to(DEV), V.to(dtype).to(DEV), s.to(DEV)


def _both(call):
    """call() under the product library and under the one with bounds checks; the record of the latter."""
    ref = call()
    torch.cuda.synchronize()
    with B.bounds_checked_library():
        assert B.kvr_debug_bounds_violation() == 0            # (clears what an earlier test may have left)
        dbg = call()
        torch.cuda.synchronize()
        worst = B.kvr_debug_bounds_violation()
    return ref, dbg, worst


def test_the_record_of_failed_checks_works():
    assert B.kvr_debug_bounds_selftest() == 5                  # product build: the index comes back unchanged
    assert B.kvr_debug_bounds_violation() == 0
    with B.bounds_checked_library():
        B.kvr_debug_bounds_violation()
        assert B.kvr_debug_bounds_selftest() == 2              # clamped to limit - 1
        assert B.kvr_debug_bounds_violation() == 199           # ... and recorded
        assert B.kvr_debug_bounds_violation() == 0             # reading clears the record


@pytest.mark.parametrize("name,heads,b,lam", [("c5", 16, None, None), ("c5", 8, 64, 1.0), ("c4", 8, None, None),
                                              ("c5", 6, 200, None), ("c5", 6, None, 0.25)])
def test_benchmark_shapes_under_bounds_checks(name, heads, b, lam):
    w = W.WORKLOADS[name]
    data = W.generate(w, heads=heads, seed=5, device=DEV)
    b = w.b if b is None else b
    lam = w.lam if lam is None else lam
    call = lambda: B.kvr_retain(data["K"], data["V"], b, lam, 1e-6, Q=data.get("Q"), s=data.get("s"))
    ref, dbg, worst = _both(call)
    assert worst == 0
    for f in ("idx_sorted", "pick_order", "pick_gain", "K_out", "V_out"):
        assert torch.equal(getattr(ref, f), getattr(dbg, f)), f


@pytest.mark.parametrize("n,b,dtype,scale", [
    (257, 2, torch.bfloat16, 1.0), (300, 128, torch.bfloat16, 1e-3), (1000, 33, torch.bfloat16, 1.0),
    (2049, 40, torch.bfloat16, 1e-3), (4096, 128, torch.bfloat16, 1e-3), (4097, 70, torch.bfloat16, 1.0),
    (8192, 256, torch.bfloat16, 1e-3), (1024, 1000, torch.bfloat16, 1.0),
    (700, 128, torch.float32, 1e-3), (2049, 128, torch.float32, 1e-3), (4096, 64, torch.float32, 1.0)])
def test_ragged_long_heads_under_bounds_checks(n, b, dtype, scale):
    K, V, s = _mk(3, n, 777 + n + b, dtype, scale)
    call = lambda: B.kvr_retain(K, V, b, 0.5, 1e-6, s=s)
    ref, dbg, worst = _both(call)
    assert worst == 0
    for f in ("idx_sorted", "pick_order", "pick_gain", "K_out", "V_out"):
        assert torch.equal(getattr(ref, f), getattr(dbg, f)), f


def test_tied_and_crowded_scores_under_bounds_checks():
    # identical rows with heavily tied scores, and gains within one percent of each other: the paths
    # with epochs that end without a pick and with full-width keys
    for n, b in ((1000, 120), (3000, 128)):
        K, V, s = _mk(2, n, 31 + n, torch.bfloat16, 1.0)
        V[:] = V[:, :1, :]
        s = torch.floor(s * 8) / 8
        ref, dbg, worst = _both(lambda: B.kvr_retain(K, V, b, 0.75, 1e-6, s=s))
        assert worst == 0 and torch.equal(ref.pick_order, dbg.pick_order)
        s2 = (1.502 + 0.005 * torch.rand((2, n), generator=torch.Generator().manual_seed(n))).to(DEV)
        ref, dbg, worst = _both(lambda: B.kvr_retain(K, V, b, 0.5, 1e-6, s=s2))
        assert worst == 0 and torch.equal(ref.pick_order, dbg.pick_order)


@pytest.mark.parametrize("n,b", [(1024, 128), (4096, 64), (2500, 100)])
def test_long_heads_with_wide_scores_under_bounds_checks(n, b):
    # log-normal scores handed in: the kernel that shrinks a long head to the tokens the score bound leaves
    # (survivor positions and tokens are range-checked), the lazy kernel on the heads it hands on
    K, V, s = _mk(5, n, 99 + n + b, torch.bfloat16, 1.0)
    s = torch.randn(s.shape, generator=torch.Generator().manual_seed(n + b)).exp().to(DEV)
    s[1] = s[1] * 0.05                                   # too tight for the bound: handed on
    ref, dbg, worst = _both(lambda: B.kvr_retain(K, V, b, 0.5, 1e-6, s=s))
    assert worst == 0
    for f in ("idx_sorted", "pick_order", "pick_gain", "K_out", "V_out"):
        assert torch.equal(getattr(ref, f), getattr(dbg, f)), f
