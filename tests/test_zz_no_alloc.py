"""kvr_retain_budgeted_static (the entry point that allocates nothing: its scratch is a static device
array of the library) against kvr_retain_budgeted, through the C-ABI, on two calls in a row, the second
with a smaller input.  Collected last: a failure here must not hide the tests before it."""
import ctypes

import pytest
import torch

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _inputs(heads, n, b_max, seed, computed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    K = torch.randn((heads, n, 128), generator=g).to(torch.bfloat16).to(DEV)
    V = torch.randn((heads, n, 128), generator=g)
    V[:, n // 2:] = V[:, : n - n // 2] + 0.05 * V[:, n // 2:]          # near-duplicate rows: the penalty matters
    V = V.to(torch.bfloat16).to(DEV)
    s = torch.rand((heads, n), generator=g).to(DEV)
    Q = torch.randn((heads, 4, 128), generator=g).to(torch.bfloat16).to(DEV) if computed else None
    n_h = torch.randint(max(b_max, n // 2), n + 1, (heads,), generator=g, dtype=torch.int32).to(DEV)
    b_h = torch.randint(b_max // 2, b_max + 1, (heads,), generator=g, dtype=torch.int32).to(DEV)
    keep = torch.zeros((heads, n), dtype=torch.uint8)
    keep[:, :3] = 1
    keep = keep.to(DEV)
    pos = (torch.arange(n, dtype=torch.int32) * 3 + 7).repeat(heads, 1).contiguous().to(DEV)
    lam_h = (0.25 + 0.5 * torch.rand((heads,), generator=g)).to(DEV)
    return dict(K=K, V=V, s=None if computed else s, Q=Q, n_h=n_h, b_h=b_h, keep=keep, pos=pos, lam_h=lam_h)


def _same(a, c, b_h, b_max):
    valid = torch.arange(b_max, device=DEV).view(1, -1) < b_h.view(-1, 1)
    assert torch.equal(a.idx_sorted, c.idx_sorted)
    assert torch.equal(a.pick_order, c.pick_order)
    assert torch.equal(a.pick_gain.view(torch.int32), c.pick_gain.view(torch.int32))      # bit for bit, padding included
    assert torch.equal(torch.where(valid, a.pos_out, 0), torch.where(valid, c.pos_out, 0))
    rows = valid.unsqueeze(-1)
    for x, y in ((a.K_out, c.K_out), (a.V_out, c.V_out)):
        assert torch.equal(torch.where(rows, x.view(torch.int16), 0), torch.where(rows, y.view(torch.int16), 0))


@pytest.mark.parametrize("computed", [False, True])
def test_static_scratch_entry_point_matches_the_one_with_a_caller_buffer(computed):
    from paper_2605_14292_amd import binding as B
    # first call: 700 heads of 192 tokens (the fused short-head kernels); second, smaller call right after it:
    # 37 heads of 600 tokens (the long-head kernel), so stale contents of the array lie beyond and beneath it
    for heads, n, b_max, lam, seed in ((700, 192, 64, 0.5, 11), (37, 600, 40, 0.5, 12), (5, 100, 16, 0.0, 13)):
        d = _inputs(heads, n, b_max, seed, computed)
        kw = dict(Q=d["Q"], s=d["s"], n_h=d["n_h"], b_h=d["b_h"], keep=d["keep"], pos=d["pos"],
                  lam_h=d["lam_h"] if lam > 0 else None)
        ref = B.kvr_retain_budgeted(d["K"], d["V"], b_max, lam, 1e-6, **kw)
        got = B.kvr_retain_budgeted_static(d["K"], d["V"], b_max, lam, 1e-6, **kw)
        torch.cuda.synchronize()
        _same(ref, got, d["b_h"], b_max)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    from paper_2605_14292_amd import binding as B
    # heads * n above the array's size: refused on the host, nothing is launched, no device memory is touched
    heads, n = 2049, 4096
    assert heads * n > B.STATIC_SCRATCH_FLOATS
    lay = B.kvr_layout(heads, n, 128, 1, n * 128, 128)
    one = torch.zeros(64, dtype=torch.int32, device=DEV)
    p = ctypes.c_void_p(one.data_ptr())
    rc = B.lib().kvr_retain_budgeted_static(p, p, None, 0, p, ctypes.byref(lay), None, None, 16, None, None, None,
                                            0.5, 1e-6, p, p, p, None, None, None, None)
    assert rc == -3 and "workspace" in B.strerror(rc)
