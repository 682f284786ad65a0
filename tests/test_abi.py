"""The C-ABI library loads, exports everything include/kvr.h declares, and
rejects bad arguments on the host before anything is launched.  No GPU."""
import ctypes
import os
import re

from paper_2605_14292_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "kvr.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvr_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert set(B.EXPORTS) == set(names)
    for nm in names:
        assert hasattr(B.lib(), nm), nm


def test_version_and_strerror():
    assert B.kvr_version() >= 1
    assert B.strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -99):
        assert isinstance(B.strerror(code), str) and B.strerror(code)


def test_debug_entry_points_of_the_product_build():
    # the product build has no bounds checks: its record is always empty (no GPU call is made)
    L = B.lib()
    worst = ctypes.c_uint32(77)
    assert L.kvr_debug_bounds_violation(ctypes.byref(worst)) == 0 and worst.value == 0
    assert L.kvr_debug_bounds_violation(None) == B.KVR_ERR_ARG
    assert L.kvr_debug_bounds_selftest(None, None) == B.KVR_ERR_ARG
    lay = _lay()
    fake = ctypes.c_void_p(0x1000)
    val = L.kvr_debug_validate_finite
    assert val(None, None, None, 0, None, ctypes.byref(lay), None) == B.KVR_ERR_ARG
    assert val(fake, None, None, 0, None, None, None) == B.KVR_ERR_ARG
    assert val(fake, None, fake, 0, None, ctypes.byref(lay), None) == B.KVR_ERR_ARG
    assert val(fake, None, fake, 257, None, ctypes.byref(lay), None) == B.KVR_ERR_UNSUPPORTED
    assert val(ctypes.c_void_p(0x1004), None, None, 0, None, ctypes.byref(lay), None) == B.KVR_ERR_ARG
    bad_d = _lay(d=64)
    assert val(fake, None, None, 0, None, ctypes.byref(bad_d), None) == B.KVR_ERR_UNSUPPORTED
    assert "finite" in B.strerror(B.KVR_ERR_NONFINITE)


def test_the_build_with_bounds_checks_exports_the_same_symbols():
    lib = ctypes.CDLL(B.BOUNDS_LIB_PATH)
    for nm in _declared():
        assert hasattr(lib, nm), nm


def _lay(heads=2, n=64, d=128, dtype=B.KVR_BF16, sh=None, st=None):
    st = d if st is None else st
    sh = n * st if sh is None else sh
    return B.kvr_layout(heads, n, d, dtype, sh, st)


def test_layout_struct_matches_header():
    assert ctypes.sizeof(B.kvr_layout) == 32


def test_argument_errors_are_host_side():
    L = B.lib()
    fake = ctypes.c_void_p(0x1000)           # never dereferenced: validation fails first
    out = ctypes.c_size_t(7)
    lay = _lay()
    assert L.kvr_workspace_bytes(ctypes.byref(lay), 16, 4, ctypes.byref(out)) == 0 and out.value == 0
    assert L.kvr_workspace_bytes(None, 16, 4, ctypes.byref(out)) == B.KVR_ERR_ARG
    bad_d = _lay(d=64)
    assert L.kvr_score(fake, fake, 1, ctypes.byref(bad_d), fake, None) == B.KVR_ERR_UNSUPPORTED
    big_n = _lay(n=8193)
    assert L.kvr_score(fake, fake, 1, ctypes.byref(big_n), fake, None) == B.KVR_ERR_UNSUPPORTED
    assert L.kvr_score(fake, fake, 0, ctypes.byref(lay), fake, None) == B.KVR_ERR_ARG
    assert L.kvr_score(fake, fake, 257, ctypes.byref(lay), fake, None) == B.KVR_ERR_UNSUPPORTED
    assert L.kvr_score(None, fake, 1, ctypes.byref(lay), fake, None) == B.KVR_ERR_ARG
    odd = ctypes.c_void_p(0x1004)
    assert L.kvr_score(odd, fake, 1, ctypes.byref(lay), fake, None) == B.KVR_ERR_ARG
    sel = L.kvr_select_greedy
    assert sel(fake, fake, ctypes.byref(lay), 0, 0.5, 1e-6, fake, None, None, None, 0, None) == B.KVR_ERR_ARG
    assert sel(fake, fake, ctypes.byref(lay), 65, 0.5, 1e-6, fake, None, None, None, 0, None) == B.KVR_ERR_ARG
    assert sel(fake, fake, ctypes.byref(lay), 8, -0.1, 1e-6, fake, None, None, None, 0, None) == B.KVR_ERR_ARG
    assert sel(fake, fake, ctypes.byref(lay), 8, float("nan"), 1e-6, fake, None, None, None, 0, None) == B.KVR_ERR_ARG
    assert sel(None, fake, ctypes.byref(lay), 8, 0.5, 1e-6, fake, None, None, None, 0, None) == B.KVR_ERR_ARG
    assert sel(fake, fake, ctypes.byref(lay), 8, 0.5, 1e-6, None, None, None, None, 0, None) == B.KVR_ERR_ARG
    short = _lay(st=64)
    assert sel(fake, fake, ctypes.byref(short), 8, 0.5, 1e-6, fake, None, None, None, 0, None) == B.KVR_ERR_ARG
    overlap = _lay(sh=100)
    assert sel(fake, fake, ctypes.byref(overlap), 8, 0.5, 1e-6, fake, None, None, None, 0, None) == B.KVR_ERR_ARG
    bad_dt = _lay(dtype=5)
    assert sel(fake, fake, ctypes.byref(bad_dt), 8, 0.5, 1e-6, fake, None, None, None, 0, None) == B.KVR_ERR_UNSUPPORTED
    cp = L.kvr_compact
    assert cp(fake, fake, ctypes.byref(lay), None, 8, fake, fake, None) == B.KVR_ERR_ARG
    assert cp(fake, None, ctypes.byref(lay), fake, 8, fake, fake, None) == B.KVR_ERR_ARG
    assert cp(None, None, ctypes.byref(lay), fake, 8, None, None, None) == B.KVR_ERR_ARG
    rt = L.kvr_retain
    # both Q and s, or neither
    assert rt(fake, fake, fake, 1, fake, ctypes.byref(lay), 8, 0.5, 1e-6, fake, fake, None, None, fake, fake, None, 0, None) == B.KVR_ERR_ARG
    assert rt(fake, fake, None, 0, None, ctypes.byref(lay), 8, 0.5, 1e-6, fake, fake, None, None, fake, fake, None, 0, None) == B.KVR_ERR_ARG
    assert rt(fake, fake, None, 0, fake, ctypes.byref(lay), 80, 0.5, 1e-6, None, fake, None, None, fake, fake, None, 0, None) == B.KVR_ERR_ARG


def test_binding_refuses_cpu_tensors():
    import pytest
    import torch
    V = torch.zeros((1, 8, 128), dtype=torch.bfloat16)
    s = torch.zeros((1, 8))
    with pytest.raises(ValueError):
        B.kvr_select_greedy(V, s, 2, 0.5)


def test_flat_mode_argument_errors_are_host_side():
    L = B.lib()
    fake = ctypes.c_void_p(0x1000)
    lay = _lay(heads=6)
    assert L.kvr_signature_flat(fake, ctypes.byref(lay), 4, fake, None) == B.KVR_ERR_ARG      # 6 % 4 != 0
    assert L.kvr_signature_flat(fake, ctypes.byref(lay), 0, fake, None) == B.KVR_ERR_ARG
    assert L.kvr_signature_flat(None, ctypes.byref(lay), 3, fake, None) == B.KVR_ERR_ARG
    assert L.kvr_compact_shared(fake, fake, ctypes.byref(lay), 4, fake, 8, fake, fake, None) == B.KVR_ERR_ARG
    assert L.kvr_compact_shared(fake, fake, ctypes.byref(lay), 3, None, 8, fake, fake, None) == B.KVR_ERR_ARG
    pl = L.kvr_score_pool
    other = ctypes.c_void_p(0x2000)
    assert pl(fake, 4, 64, 7, 0, fake, None) == B.KVR_ERR_ARG        # in place
    assert pl(fake, 4, 64, 6, 0, other, None) == B.KVR_ERR_ARG       # even window
    assert pl(fake, 4, 64, 65, 0, other, None) == B.KVR_ERR_ARG      # window too wide
    assert pl(fake, 4, 64, 7, 2, other, None) == B.KVR_ERR_ARG       # unknown mode
    assert pl(fake, 0, 64, 7, 0, other, None) == B.KVR_ERR_ARG
    assert pl(None, 4, 64, 7, 0, other, None) == B.KVR_ERR_ARG
    sp = L.kvr_score_prior
    assert sp(None, ctypes.byref(lay), fake, 0.5, 1e-6, fake, None) == B.KVR_ERR_ARG
    assert sp(fake, ctypes.byref(lay), None, 0.5, 1e-6, fake, None) == B.KVR_ERR_ARG
    assert sp(fake, ctypes.byref(lay), fake, float("nan"), 1e-6, fake, None) == B.KVR_ERR_ARG
    assert sp(fake, ctypes.byref(lay), fake, 0.5, -1.0, fake, None) == B.KVR_ERR_ARG
    ci = L.kvr_compact_inplace
    assert ci(fake, fake, ctypes.byref(lay), 4, fake, 8, None, None) == B.KVR_ERR_ARG      # 6 % 4 != 0
    assert ci(fake, fake, ctypes.byref(lay), 1, None, 8, None, None) == B.KVR_ERR_ARG      # no index list
    assert ci(None, None, ctypes.byref(lay), 1, fake, 8, None, None) == B.KVR_ERR_ARG      # nothing to move
    assert ci(fake, fake, ctypes.byref(lay), 1, fake, 65, None, None) == B.KVR_ERR_ARG     # b > n
    assert ci(ctypes.c_void_p(0x1004), fake, ctypes.byref(lay), 1, fake, 8, None, None) == B.KVR_ERR_ARG
    rf = L.kvr_retain_flat
    assert rf(fake, fake, fake, ctypes.byref(lay), 3, 8, 0.5, 1e-6, None, fake, None, None, fake, fake, None) == B.KVR_ERR_ARG
    assert rf(fake, fake, fake, ctypes.byref(lay), 4, 8, 0.5, 1e-6, fake, fake, None, None, fake, fake, None) == B.KVR_ERR_ARG
    assert rf(fake, fake, fake, ctypes.byref(lay), 3, 65, 0.5, 1e-6, fake, fake, None, None, fake, fake, None) == B.KVR_ERR_ARG
    assert rf(fake, fake, None, ctypes.byref(lay), 3, 8, 0.5, 1e-6, fake, fake, None, None, fake, fake, None) == B.KVR_ERR_ARG


def test_budgeted_argument_errors_are_host_side():
    L = B.lib()
    fake = ctypes.c_void_p(0x1000)
    lay = _lay()
    rb = L.kvr_retain_budgeted
    ok_tail = (fake, fake, fake, fake, fake, fake, None, None)        # s_work .. stream
    assert rb(fake, fake, None, 0, fake, ctypes.byref(lay), None, None, 65, None, None, None, 0.5, 1e-6, *ok_tail) == B.KVR_ERR_ARG
    assert rb(fake, fake, None, 0, None, ctypes.byref(lay), None, None, 8, None, None, None, 0.5, 1e-6, *ok_tail) == B.KVR_ERR_ARG
    assert rb(fake, fake, fake, 1, fake, ctypes.byref(lay), None, None, 8, None, None, None, 0.5, 1e-6, *ok_tail) == B.KVR_ERR_ARG
    assert rb(fake, fake, None, 0, fake, ctypes.byref(lay), None, None, 8, None, None, None, 0.5, 1e-6,
              None, fake, fake, fake, fake, fake, None, None) == B.KVR_ERR_ARG                       # no s_work
    assert rb(fake, fake, None, 0, fake, ctypes.byref(lay), None, None, 8, None, None, None, 0.5, 1e-6,
              fake, fake, None, fake, fake, fake, None, None) == B.KVR_ERR_ARG                       # no pick_order
    assert rb(fake, fake, None, 0, fake, ctypes.byref(lay), None, None, 8, None, None, None, 0.5, 1e-6,
              fake, fake, fake, fake, fake, fake, fake, None) == B.KVR_ERR_ARG                       # pos_out without pos_in
    assert rb(fake, fake, None, 0, fake, ctypes.byref(lay), None, None, 8, None, None, fake, 0.0, 1e-6, *ok_tail) == B.KVR_ERR_ARG   # lambda_h needs lambda > 0

