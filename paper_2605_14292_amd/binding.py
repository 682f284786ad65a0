"""ctypes binding of libkvr.so: argument marshalling only.

Every function has the name and the meaning of the C entry point declared in
include/kvr.h; tensors are torch device tensors used as plain device buffers.
The library is required: importing this module without a built libkvr.so, or
calling it without a GPU, raises.
"""
from __future__ import annotations

import contextlib
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvr.so")

KVR_F32, KVR_BF16 = 0, 1
KVR_OK, KVR_ERR_ARG, KVR_ERR_UNSUPPORTED, KVR_ERR_WORKSPACE, KVR_ERR_HIP, KVR_ERR_NONFINITE = 0, -1, -2, -3, -4, -5

EXPORTS = ("kvr_version", "kvr_strerror", "kvr_workspace_bytes", "kvr_score",
           "kvr_select_greedy", "kvr_compact", "kvr_retain",
           "kvr_signature_flat", "kvr_compact_shared", "kvr_compact_inplace", "kvr_score_prior", "kvr_score_pool", "kvr_retain_flat",
           "kvr_retain_budgeted", "kvr_retain_budgeted_static", "kvr_debug_bounds_violation",
           "kvr_debug_bounds_selftest", "kvr_debug_validate_finite")


class kvr_layout(ctypes.Structure):
    _fields_ = [("heads", ctypes.c_int32), ("n", ctypes.c_int32), ("d", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("stride_head", ctypes.c_int64),
                ("stride_tok", ctypes.c_int64)]


class KvrError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


def _load(path: str = LIB_PATH) -> ctypes.CDLL:
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is missing: build it with `python -m paper_2605_14292_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(path)
    vp, i32, f32 = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    lp = ctypes.POINTER(kvr_layout)
    lib.kvr_version.restype = i32
    lib.kvr_strerror.restype = ctypes.c_char_p
    lib.kvr_strerror.argtypes = [i32]
    lib.kvr_workspace_bytes.restype = i32
    lib.kvr_workspace_bytes.argtypes = [lp, i32, i32, ctypes.POINTER(ctypes.c_size_t)]
    lib.kvr_score.restype = i32
    lib.kvr_score.argtypes = [vp, vp, i32, lp, vp, vp]
    lib.kvr_select_greedy.restype = i32
    lib.kvr_select_greedy.argtypes = [vp, vp, lp, i32, f32, f32, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.kvr_compact.restype = i32
    lib.kvr_compact.argtypes = [vp, vp, lp, vp, i32, vp, vp, vp]
    lib.kvr_retain.restype = i32
    lib.kvr_retain.argtypes = [vp, vp, vp, i32, vp, lp, i32, f32, f32, vp, vp, vp, vp, vp, vp, vp,
                               ctypes.c_size_t, vp]
    lib.kvr_signature_flat.restype = i32
    lib.kvr_signature_flat.argtypes = [vp, lp, i32, vp, vp]
    lib.kvr_compact_shared.restype = i32
    lib.kvr_compact_shared.argtypes = [vp, vp, lp, i32, vp, i32, vp, vp, vp]
    lib.kvr_score_pool.restype = i32
    lib.kvr_score_pool.argtypes = [vp, i32, i32, i32, i32, vp, vp]
    lib.kvr_score_prior.restype = i32
    lib.kvr_score_prior.argtypes = [vp, lp, vp, f32, f32, vp, vp]
    lib.kvr_compact_inplace.restype = i32
    lib.kvr_compact_inplace.argtypes = [vp, vp, lp, i32, vp, i32, vp, vp]
    lib.kvr_retain_flat.restype = i32
    lib.kvr_retain_flat.argtypes = [vp, vp, vp, lp, i32, i32, f32, f32, vp, vp, vp, vp, vp, vp, vp]
    lib.kvr_retain_budgeted.restype = i32
    lib.kvr_retain_budgeted.argtypes = [vp, vp, vp, i32, vp, lp, vp, vp, i32, vp, vp, vp, f32, f32,
                                        vp, vp, vp, vp, vp, vp, vp, vp]
    lib.kvr_retain_budgeted_static.restype = i32
    lib.kvr_retain_budgeted_static.argtypes = [vp, vp, vp, i32, vp, lp, vp, vp, i32, vp, vp, vp, f32, f32,
                                               vp, vp, vp, vp, vp, vp, vp]
    lib.kvr_debug_bounds_violation.restype = i32
    lib.kvr_debug_bounds_violation.argtypes = [ctypes.POINTER(ctypes.c_uint32)]
    lib.kvr_debug_bounds_selftest.restype = i32
    lib.kvr_debug_bounds_selftest.argtypes = [vp, vp]
    lib.kvr_debug_validate_finite.restype = i32
    lib.kvr_debug_validate_finite.argtypes = [vp, vp, vp, i32, vp, lp, vp]
    return lib


_lib = _load()
BOUNDS_LIB_PATH = os.path.join(os.path.dirname(LIB_PATH), "libkvr_bounds.so")


def lib() -> ctypes.CDLL:
    return _lib


@contextlib.contextmanager
def bounds_checked_library():
    """Routes every call of this module through the debug build with bounds checks (libkvr_bounds.so, built by
    `python -m paper_2605_14292_amd.build`) for the duration of the block."""
    global _lib
    product, _lib = _lib, _load(BOUNDS_LIB_PATH)
    try:
        yield _lib
    finally:
        _lib = product


def kvr_debug_validate_finite(K=None, V=None, Q=None, s=None, lay=None, stream=None) -> bool:
    """True when K, V, Q and s (those given) hold only finite values.  Synchronises the stream."""
    rows = K if K is not None else V
    _need_cuda(K, V, Q, s)
    lay = layout_of(rows) if lay is None else lay
    for t in (K, V):
        if t is not None and (t.shape[0], t.shape[1], t.stride(0), t.stride(1)) != (lay.heads, lay.n, lay.stride_head, lay.stride_tok):
            raise ValueError("K and V must share the layout")
    if s is not None and (tuple(s.shape) != (lay.heads, lay.n) or not s.is_contiguous() or s.dtype != torch.float32):
        raise ValueError("s must be a dense fp32 [heads, n] tensor")
    if Q is not None and (Q.shape[0] != lay.heads or not Q.is_contiguous()):
        raise ValueError("Q must be a dense [heads, G, d] tensor")
    G = 0 if Q is None else int(Q.shape[1])
    rc = _lib.kvr_debug_validate_finite(_ptr(K), _ptr(V), _ptr(Q), G, _ptr(s), ctypes.byref(lay), _stream(stream))
    if rc == KVR_ERR_NONFINITE:
        return False
    _check(rc, "kvr_debug_validate_finite")
    return True


def kvr_debug_bounds_selftest(stream=None) -> int:
    """The index that the range check made of 5 with the limit 3: 2 with bounds checks, 5 without."""
    import torch
    out = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    _check(_lib.kvr_debug_bounds_selftest(_ptr(out), _stream(stream)), "kvr_debug_bounds_selftest")
    torch.cuda.synchronize()
    return int(out.item())


def kvr_debug_bounds_violation() -> int:
    """Largest id of a bounds check that failed since the last call (0: none; always 0 in the product build)."""
    worst = ctypes.c_uint32(0xdeadbeef)
    _check(_lib.kvr_debug_bounds_violation(ctypes.byref(worst)), "kvr_debug_bounds_violation")
    return int(worst.value)


def strerror(status: int) -> str:
    return _lib.kvr_strerror(int(status)).decode()


def kvr_version() -> int:
    return int(_lib.kvr_version())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def layout_of(x: torch.Tensor) -> kvr_layout:
    """Layout of a [heads, n, d] device tensor (last dim contiguous)."""
    if x.dim() != 3 or x.stride(2) != 1:
        raise ValueError("expected a [heads, n, d] tensor with contiguous d")
    if x.dtype == torch.bfloat16:
        dt = KVR_BF16
    elif x.dtype == torch.float32:
        dt = KVR_F32
    else:
        raise ValueError("dtype must be bfloat16 or float32")
    return kvr_layout(x.shape[0], x.shape[1], x.shape[2], dt, x.stride(0), x.stride(1))


def _need_cuda(*ts):
    for t in ts:
        if t is not None and not t.is_cuda:
            raise ValueError("kvr takes device tensors only (no CPU fallback exists)")


def _check(rc: int, where: str):
    if rc != KVR_OK:
        raise KvrError(rc, where)


def kvr_workspace_bytes(lay: kvr_layout, b: int, G: int) -> int:
    out = ctypes.c_size_t(0)
    _check(_lib.kvr_workspace_bytes(ctypes.byref(lay), b, G, ctypes.byref(out)), "kvr_workspace_bytes")
    return int(out.value)


def kvr_score(K, Q, s_out=None, stream=None):
    _need_cuda(K, Q, s_out)
    lay = layout_of(K)
    G = Q.shape[1]
    if s_out is None:
        s_out = torch.empty((lay.heads, lay.n), dtype=torch.float32, device=K.device)
    _check(_lib.kvr_score(_ptr(K), _ptr(Q), G, ctypes.byref(lay), _ptr(s_out), _stream(stream)),
           "kvr_score")
    return s_out


def kvr_select_greedy(V, s, b, lam, eps=1e-6, idx_sorted=None, pick_order=None, pick_gain=None,
                      want_trace=True, stream=None, lay=None):
    _need_cuda(V, s, idx_sorted, pick_order, pick_gain)
    if lay is None:
        lay = layout_of(V)
    dev = s.device
    if idx_sorted is None:
        idx_sorted = torch.empty((lay.heads, b), dtype=torch.int32, device=dev)
    if want_trace:
        if pick_order is None:
            pick_order = torch.empty((lay.heads, b), dtype=torch.int32, device=dev)
        if pick_gain is None:
            pick_gain = torch.empty((lay.heads, b), dtype=torch.float32, device=dev)
    _check(_lib.kvr_select_greedy(_ptr(V), _ptr(s), ctypes.byref(lay), b, lam, eps,
                                  _ptr(idx_sorted), _ptr(pick_order), _ptr(pick_gain),
                                  None, 0, _stream(stream)), "kvr_select_greedy")
    return idx_sorted, pick_order, pick_gain


def kvr_compact(K, V, idx, K_out=None, V_out=None, stream=None):
    _need_cuda(K, V, idx, K_out, V_out)
    ref = K if K is not None else V
    lay = layout_of(ref)
    b = idx.shape[1]
    if K is not None and K_out is None:
        K_out = torch.empty((lay.heads, b, lay.d), dtype=K.dtype, device=K.device)
    if V is not None and V_out is None:
        V_out = torch.empty((lay.heads, b, lay.d), dtype=V.dtype, device=V.device)
    _check(_lib.kvr_compact(_ptr(K), _ptr(V), ctypes.byref(lay), _ptr(idx), b, _ptr(K_out),
                            _ptr(V_out), _stream(stream)), "kvr_compact")
    return K_out, V_out


class RetainBuffers:
    """Preallocated outputs of kvr_retain for one shape (so a timed loop
    allocates nothing)."""

    def __init__(self, heads, n, b, d, dtype, device, computed_scores, want_trace=True):
        self.idx_sorted = torch.empty((heads, b), dtype=torch.int32, device=device)
        self.pick_order = torch.empty((heads, b), dtype=torch.int32, device=device) if want_trace else None
        self.pick_gain = torch.empty((heads, b), dtype=torch.float32, device=device) if want_trace else None
        self.K_out = torch.empty((heads, b, d), dtype=dtype, device=device)
        self.V_out = torch.empty((heads, b, d), dtype=dtype, device=device)
        self.s_out = torch.empty((heads, n), dtype=torch.float32, device=device) if computed_scores else None


def kvr_retain(K, V, b, lam, eps=1e-6, Q=None, s=None, out: RetainBuffers | None = None,
               want_trace=True, stream=None):
    _need_cuda(K, V, Q, s)
    lay = layout_of(K)
    if layout_of(V).stride_head != lay.stride_head or layout_of(V).stride_tok != lay.stride_tok:
        raise ValueError("K and V must share one layout")
    if out is None:
        out = RetainBuffers(lay.heads, lay.n, b, lay.d, K.dtype, K.device, Q is not None, want_trace)
    G = 0 if Q is None else Q.shape[1]
    _check(_lib.kvr_retain(_ptr(K), _ptr(V), _ptr(Q), G, _ptr(s), ctypes.byref(lay), b, lam, eps,
                           _ptr(out.s_out), _ptr(out.idx_sorted), _ptr(out.pick_order),
                           _ptr(out.pick_gain), _ptr(out.K_out), _ptr(out.V_out), None, 0,
                           _stream(stream)), "kvr_retain")
    return out


def kvr_signature_flat(V, group, u_out=None, stream=None):
    _need_cuda(V, u_out)
    lay = layout_of(V)
    if u_out is None:
        u_out = torch.empty((lay.heads // group, lay.n, lay.d), dtype=torch.float32, device=V.device)
    _check(_lib.kvr_signature_flat(_ptr(V), ctypes.byref(lay), group, _ptr(u_out), _stream(stream)),
           "kvr_signature_flat")
    return u_out


def kvr_compact_shared(K, V, idx, group, K_out=None, V_out=None, stream=None):
    _need_cuda(K, V, idx, K_out, V_out)
    ref = K if K is not None else V
    lay = layout_of(ref)
    b = idx.shape[1]
    if K is not None and K_out is None:
        K_out = torch.empty((lay.heads, b, lay.d), dtype=K.dtype, device=K.device)
    if V is not None and V_out is None:
        V_out = torch.empty((lay.heads, b, lay.d), dtype=V.dtype, device=V.device)
    _check(_lib.kvr_compact_shared(_ptr(K), _ptr(V), ctypes.byref(lay), group, _ptr(idx), b,
                                   _ptr(K_out), _ptr(V_out), _stream(stream)), "kvr_compact_shared")
    return K_out, V_out


KVR_POOL_MAX, KVR_POOL_MEAN = 0, 1


def kvr_score_pool(s, kernel, mode=KVR_POOL_MAX, s_out=None, stream=None):
    """Max or mean of each score row over a centred window of `kernel` (odd) tokens."""
    _need_cuda(s, s_out)
    if s.dtype != torch.float32 or s.dim() != 2 or not s.is_contiguous():
        raise ValueError("s must be a contiguous float32 [heads, n] tensor")
    if s_out is None:
        s_out = torch.empty_like(s)
    _check(_lib.kvr_score_pool(_ptr(s), s.shape[0], s.shape[1], kernel, mode, _ptr(s_out), _stream(stream)),
           "kvr_score_pool")
    return s_out


def kvr_score_prior(V, s, lam_p, eps=1e-6, s_out=None, stream=None):
    """s + lam_p * cos(V_i, mean row of the head): the modular prior the paper rejected."""
    _need_cuda(V, s, s_out)
    lay = layout_of(V)
    if s.dtype != torch.float32 or tuple(s.shape) != (lay.heads, lay.n) or not s.is_contiguous():
        raise ValueError("s must be a contiguous float32 [heads, n] tensor")
    if s_out is None:
        s_out = torch.empty_like(s)
    _check(_lib.kvr_score_prior(_ptr(V), ctypes.byref(lay), _ptr(s), lam_p, eps, _ptr(s_out), _stream(stream)),
           "kvr_score_prior")
    return s_out


def kvr_compact_inplace(K, V, idx, group=1, pos=None, stream=None):
    """Moves the kept rows to the front of each head inside K and V (and pos) themselves."""
    _need_cuda(K, V, idx, pos)
    ref = K if K is not None else V
    if ref is None:
        raise ValueError("kvr_compact_inplace needs K or V (the layout comes from them)")
    lay = layout_of(ref)
    if pos is not None and (pos.dtype != torch.int32 or tuple(pos.shape) != (lay.heads, lay.n)
                            or not pos.is_contiguous()):
        raise ValueError("pos must be a contiguous int32 [heads, n] tensor")
    _check(_lib.kvr_compact_inplace(_ptr(K), _ptr(V), ctypes.byref(lay), group, _ptr(idx), idx.shape[1],
                                    _ptr(pos), _stream(stream)), "kvr_compact_inplace")


class FlatBuffers:
    """Preallocated outputs of kvr_retain_flat for one shape."""

    def __init__(self, heads, group, n, b, d, dtype, device, want_trace=True):
        seqs = heads // group
        self.u_out = torch.empty((seqs, n, d), dtype=torch.float32, device=device)
        self.idx_sorted = torch.empty((seqs, b), dtype=torch.int32, device=device)
        self.pick_order = torch.empty((seqs, b), dtype=torch.int32, device=device) if want_trace else None
        self.pick_gain = torch.empty((seqs, b), dtype=torch.float32, device=device) if want_trace else None
        self.K_out = torch.empty((heads, b, d), dtype=dtype, device=device)
        self.V_out = torch.empty((heads, b, d), dtype=dtype, device=device)


def kvr_retain_flat(K, V, s, group, b, lam, eps=1e-6, out: FlatBuffers | None = None,
                    want_trace=True, stream=None):
    _need_cuda(K, V, s)
    lay = layout_of(K)
    if layout_of(V).stride_head != lay.stride_head or layout_of(V).stride_tok != lay.stride_tok:
        raise ValueError("K and V must share one layout")
    if out is None:
        out = FlatBuffers(lay.heads, group, lay.n, b, lay.d, K.dtype, K.device, want_trace)
    _check(_lib.kvr_retain_flat(_ptr(K), _ptr(V), _ptr(s), ctypes.byref(lay), group, b, lam, eps,
                                _ptr(out.u_out), _ptr(out.idx_sorted), _ptr(out.pick_order),
                                _ptr(out.pick_gain), _ptr(out.K_out), _ptr(out.V_out),
                                _stream(stream)), "kvr_retain_flat")
    return out


class BudgetBuffers:
    """Preallocated outputs of kvr_retain_budgeted for one shape."""

    def __init__(self, heads, n, b_max, d, dtype, device, with_pos=False):
        self.s_work = torch.empty((heads, n), dtype=torch.float32, device=device)
        self.idx_sorted = torch.empty((heads, b_max), dtype=torch.int32, device=device)
        self.pick_order = torch.empty((heads, b_max), dtype=torch.int32, device=device)
        self.pick_gain = torch.empty((heads, b_max), dtype=torch.float32, device=device)
        self.K_out = torch.zeros((heads, b_max, d), dtype=dtype, device=device)
        self.V_out = torch.zeros((heads, b_max, d), dtype=dtype, device=device)
        self.pos_out = torch.empty((heads, b_max), dtype=torch.int32, device=device) if with_pos else None


def kvr_retain_budgeted(K, V, b_max, lam, eps=1e-6, Q=None, s=None, n_h=None, b_h=None, keep=None,
                        pos=None, lam_h=None, out: BudgetBuffers | None = None, stream=None):
    _need_cuda(K, V, Q, s, n_h, b_h, keep, pos, lam_h)
    lay = layout_of(K)
    if layout_of(V).stride_head != lay.stride_head or layout_of(V).stride_tok != lay.stride_tok:
        raise ValueError("K and V must share one layout")
    for t, dt in ((n_h, torch.int32), (b_h, torch.int32), (keep, torch.uint8), (pos, torch.int32),
                  (lam_h, torch.float32)):
        if t is not None and (t.dtype != dt or not t.is_contiguous()):
            raise ValueError("n_h, b_h, pos must be contiguous int32 and keep contiguous uint8")
    if out is None:
        out = BudgetBuffers(lay.heads, lay.n, b_max, lay.d, K.dtype, K.device, pos is not None)
    G = 0 if Q is None else Q.shape[1]
    _check(_lib.kvr_retain_budgeted(_ptr(K), _ptr(V), _ptr(Q), G, _ptr(s), ctypes.byref(lay), _ptr(n_h),
                                    _ptr(b_h), b_max, _ptr(keep), _ptr(pos), _ptr(lam_h), lam, eps, _ptr(out.s_work),
                                    _ptr(out.idx_sorted), _ptr(out.pick_order), _ptr(out.pick_gain),
                                    _ptr(out.K_out), _ptr(out.V_out), _ptr(out.pos_out), _stream(stream)),
           "kvr_retain_budgeted")
    return out


STATIC_SCRATCH_FLOATS = 8 << 20


def kvr_retain_budgeted_static(K, V, b_max, lam, eps=1e-6, Q=None, s=None, n_h=None, b_h=None, keep=None,
                               pos=None, lam_h=None, out: BudgetBuffers | None = None, stream=None):
    """kvr_retain_budgeted without the s_work argument: the adjusted scores live in the library's static
    device array (heads * n <= STATIC_SCRATCH_FLOATS); the C call allocates nothing.  `out.s_work` is not
    written."""
    _need_cuda(K, V, Q, s, n_h, b_h, keep, pos, lam_h)
    lay = layout_of(K)
    if layout_of(V).stride_head != lay.stride_head or layout_of(V).stride_tok != lay.stride_tok:
        raise ValueError("K and V must share one layout")
    for t, dt in ((n_h, torch.int32), (b_h, torch.int32), (keep, torch.uint8), (pos, torch.int32),
                  (lam_h, torch.float32)):
        if t is not None and (t.dtype != dt or not t.is_contiguous()):
            raise ValueError("n_h, b_h, pos must be contiguous int32 and keep contiguous uint8")
    if out is None:
        out = BudgetBuffers(lay.heads, lay.n, b_max, lay.d, K.dtype, K.device, pos is not None)
    G = 0 if Q is None else Q.shape[1]
    _check(_lib.kvr_retain_budgeted_static(_ptr(K), _ptr(V), _ptr(Q), G, _ptr(s), ctypes.byref(lay), _ptr(n_h),
                                           _ptr(b_h), b_max, _ptr(keep), _ptr(pos), _ptr(lam_h), lam, eps,
                                           _ptr(out.idx_sorted), _ptr(out.pick_order), _ptr(out.pick_gain),
                                           _ptr(out.K_out), _ptr(out.V_out), _ptr(out.pos_out), _stream(stream)),
           "kvr_retain_budgeted_static")
    return out
