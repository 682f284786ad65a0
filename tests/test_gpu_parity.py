"""Parity of the HIP path (through the C-ABI) with the fp64 oracle on the five
benchmark configurations and on edge cases.  Needs an MI355X."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import alpha_oracle as O
from paper_2605_14292_amd import workloads as W
import parity_util as P

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def B():
    from paper_2605_14292_amd import binding
    return binding


def _bits(t):
    t = t.detach().cpu().contiguous()
    return t.view(torch.int16).numpy() if t.dtype == torch.bfloat16 else t.view(torch.int32).numpy()


def _check_heads(w, data, out, b, lam, eps, heads):
    """Element-by-element comparison for the listed heads of a workload run."""
    reports = []
    for h in heads:
        K64, V64 = W.to_f64(data["K"][h]), W.to_f64(data["V"][h])
        if "Q" in data:
            s64 = O.score_softmax_mean(K64, W.to_f64(data["Q"][h]))
            P.check_scores(out.s_out[h].cpu().numpy(), s64)
        else:
            s64 = W.to_f64(data["s"][h])
        order = out.pick_order[h].cpu().numpy()
        gain = out.pick_gain[h].cpu().numpy()
        idx = out.idx_sorted[h].cpu().numpy()
        reports.append(P.check_head(s64, V64, b, lam, eps, order, gain, idx))
        # compaction: bit-exact rows at the HIP path's own (validated) index set
        np.testing.assert_array_equal(_bits(out.K_out[h]), O.compact(_bits(data["K"][h]), idx))
        np.testing.assert_array_equal(_bits(out.V_out[h]), O.compact(_bits(data["V"][h]), idx))
    return P.summarize(reports)


def _run(w, data, b=None, lam=None, eps=1e-6):
    b = w.b if b is None else b
    lam = w.lam if lam is None else lam
    out = B().kvr_retain(data["K"], data["V"], b, lam, eps, Q=data.get("Q"), s=data.get("s"))
    torch.cuda.synchronize()
    return out, b, lam


@pytest.mark.parametrize("name,heads", [("c1", 1), ("c2", 112), ("c3", 192), ("c3", 320), ("c5", 24), ("c4", 6)])
def test_config_small_slice_every_head(name, heads):
    w = W.WORKLOADS[name]
    data = W.generate(w, heads=heads, seed=0, device=DEV)
    out, b, lam = _run(w, data)
    rep = _check_heads(w, data, out, b, lam, 1e-6, range(heads))
    print(f"\n[{name}] {rep}")
    assert rep["heads"] == heads


@pytest.mark.parametrize("lam", [0.0, 0.25, 0.5, 1.0])
@pytest.mark.parametrize("b", [128, 64])
def test_c5_lambda_sweep(lam, b):
    w = W.WORKLOADS["c5"]
    data = W.generate(w, heads=16, seed=1, device=DEV)
    out, b, lam = _run(w, data, b=b, lam=lam)
    rep = _check_heads(w, data, out, b, lam, 1e-6, range(16))
    print(f"\n[c5 lam={lam} b={b}] {rep}")
    if lam == 0.0:
        # exactly the stable top-b of the scores the HIP path itself produced
        s = out.s_out.cpu().numpy()
        for h in range(16):
            want = np.sort(np.argsort(-s[h], kind="stable")[:b])
            np.testing.assert_array_equal(out.idx_sorted[h].cpu().numpy(), want)


# near-tie flips a full-size sample may show (picks of the HIP path that are not the fp64 argmax but within
# 1e-5 of it): the oracle itself sees 10-20 such near-ties per 64 long heads; none has flipped so far
MAX_NEAR_TIE_FLIPS = 8


@pytest.mark.parametrize("name,sample,b,lam", [
    ("c3", 128, None, None), ("c2", 112, None, None), ("c4", 64, None, None),
    ("c5", 64, 128, 0.5), ("c5", 64, 64, 0.5), ("c5", 64, 128, 0.25), ("c5", 64, 128, 1.0), ("c5", 64, 128, 0.0),
    ("c5", 64, 64, 0.0), ("c5", 64, 64, 1.0)])
def test_config_full_size_sampled_heads(name, sample, b, lam):
    """The launch configuration the benchmark times: all heads resident in HBM,
    a fixed random sample of heads checked element by element."""
    _full_size_sampled(W.WORKLOADS[name], sample, b, lam)


def _full_size_sampled(w, sample, b, lam):
    name = w.name
    data = W.generate(w, seed=0, device=DEV)
    out, b, lam = _run(w, data, b=b, lam=lam)
    rng = np.random.default_rng(7)
    heads = sorted(rng.choice(w.heads, size=min(sample, w.heads), replace=False).tolist())
    rep = _check_heads(w, data, out, b, lam, 1e-6, heads)
    print(f"\n[{name} full, {w.heads} heads, b={b}, lambda={lam}, scores {w.scores}] {rep}")
    assert rep["near_ties"] <= MAX_NEAR_TIE_FLIPS
    if lam == 0.0:                               # exactly the stable top-b of the scores the HIP path itself produced
        s = out.s_out.cpu().numpy()
        for h in heads:
            np.testing.assert_array_equal(out.idx_sorted[h].cpu().numpy(), np.sort(np.argsort(-s[h], kind="stable")[:b]))
    # properties that hold at any size, on every head
    idx = out.idx_sorted.cpu().numpy()
    assert idx.min() >= 0 and idx.max() < w.n
    assert np.all(np.diff(idx, axis=1) > 0)
    po = np.sort(out.pick_order.cpu().numpy(), axis=1)
    np.testing.assert_array_equal(po, idx)
    g = out.pick_gain.cpu().numpy()
    assert np.all(np.diff(g, axis=1) <= 0)


@pytest.mark.parametrize("name,b,lam", [("c4", 128, 0.5), ("c5", 128, 0.5), ("c5", 64, 1.0), ("c5", 128, 0.25)])
def test_long_configs_with_scores_handed_in_full_size(name, b, lam):
    """The other reading of c4 and c5 (the configurations do not say where the scores come from): log-normal scores
    handed in, as in c3.  Their spread exceeds lambda, so the score bound removes most of a head before any row is read."""
    w = W.WORKLOADS[name]
    _full_size_sampled(dataclasses.replace(w, scores="given", G=1), 64, b, lam)


@pytest.mark.parametrize("n,b,lam", [(257, 2, 0.5), (300, 64, 0.5), (700, 65, 0.25), (1024, 128, 0.5), (1025, 17, 1.0),
                                     (2047, 128, 0.5), (2049, 40, 0.3), (3001, 100, 0.5), (4096, 128, 0.5), (4096, 64, 2.0)])
def test_long_heads_with_wide_scores_shrink_to_their_candidates(n, b, lam):
    """Scores handed in that spread by more than lambda: the score bound leaves a short head, which one kernel
    finishes; heads that stay too large (scores tighter than lambda, a bound that removes too little) and heads
    with fewer than b candidates left (most scores -inf) are handed on in the same launch.  Every head is compared
    with the oracle pick by pick; the selection-only entry point must agree with the fused one."""
    h = 9
    g = torch.Generator().manual_seed(77 * n + b)
    K = torch.randn((h, n, 128), generator=g).to(torch.bfloat16)
    V = torch.randn((h, n, 128), generator=g)
    V[:, n // 3: n // 3 + n // 4] = V[:, : n // 4] + 0.05 * V[:, n // 3: n // 3 + n // 4]      # near-duplicates of earlier tokens
    V = V.to(torch.bfloat16)
    s = torch.randn((h, n), generator=g).exp()                      # log-normal(0, 1)
    s[1] = 0.3 + 0.01 * torch.rand((n,), generator=g)               # spread far below lambda: nothing can go
    s[2] = s[2] * 0.2                                               # a bound that removes too little
    s[3] = torch.floor(s[3] * 2) / 2                                # ties, also at the threshold
    s[4, : n - max(b // 2, 1)] = float("-inf")                      # fewer candidates than the budget
    s[5] = -s[5]                                                    # negative scores
    s[6] = s[6] * 100                                               # the bound leaves little more than the b best
    s = s.to(torch.float32)
    K, V, s = K.to(DEV), V.to(DEV), s.to(DEV)
    out = B().kvr_retain(K, V, b, lam, 1e-6, s=s)
    sel_idx, sel_order, sel_gain = B().kvr_select_greedy(V, s, b, lam, 1e-6)
    torch.cuda.synchronize()
    heads = [hh for hh in range(h) if hh != 4]
    _check_heads(W.WORKLOADS["c3"], {"K": K, "V": V, "s": s}, out, b, lam, 1e-6, heads)
    idx = out.idx_sorted.cpu().numpy()
    assert idx.min() >= 0 and idx.max() < n and np.all(np.diff(idx, axis=1) > 0)     # head 4 too: distinct, in range
    np.testing.assert_array_equal(sel_idx.cpu().numpy()[heads], idx[heads])
    np.testing.assert_array_equal(sel_order.cpu().numpy()[heads], out.pick_order.cpu().numpy()[heads])
    np.testing.assert_array_equal(_bits(sel_gain)[heads], _bits(out.pick_gain)[heads])


@pytest.mark.parametrize("scale", [0.01, 0.2])
def test_c3_shape_with_scores_far_below_lambda(scale):
    """c3's launch with its given scores scaled down: the score bound removes nothing (0.01) or too little
    (0.2), so the heads leave the reduced-footprint kernel for the full-size one, most of them before anything is
    computed; the picks must not care which kernel made them."""
    w = W.WORKLOADS["c3"]
    data = W.generate(w, seed=0, device=DEV)
    data["s"] = (data["s"] * scale).contiguous()
    out, b, lam = _run(w, data)
    rng = np.random.default_rng(9)
    heads = sorted(rng.choice(w.heads, size=64, replace=False).tolist())
    rep = _check_heads(w, data, out, b, lam, 1e-6, heads)
    print(f"\n[c3 scores x {scale}] {rep}")
    assert rep["near_ties"] <= MAX_NEAR_TIE_FLIPS
    idx = out.idx_sorted.cpu().numpy()
    assert idx.min() >= 0 and idx.max() < w.n and np.all(np.diff(idx, axis=1) > 0)
    np.testing.assert_array_equal(np.sort(out.pick_order.cpu().numpy(), axis=1), idx)


def _mk(h, n, seed, dtype=torch.bfloat16, d=128):
    g = torch.Generator(device="cpu").manual_seed(seed)
    K = torch.randn((h, n, d), generator=g).to(dtype)
    V = torch.randn((h, n, d), generator=g).to(dtype)
    s = torch.rand((h, n), generator=g)
    return K.to(DEV), V.to(DEV), s.to(DEV)


@pytest.mark.parametrize("n,b", [(1, 1), (2, 2), (17, 5), (77, 77), (193, 64), (257, 1), (300, 299),
                                 (1000, 33), (2049, 40), (4097, 70), (6000, 130), (8192, 256)])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_ragged_sizes(n, b, dtype):
    K, V, s = _mk(3, n, 1000 + n, dtype)
    data = {"K": K, "V": V, "s": s}
    out = B().kvr_retain(K, V, b, 0.5, 1e-6, s=s)
    torch.cuda.synchronize()
    w = W.WORKLOADS["c3"]
    rep = _check_heads(w, data, out, b, 0.5, 1e-6, range(3))
    assert rep["heads"] == 3


@pytest.mark.parametrize("reps", [1, 23])
@pytest.mark.parametrize("n,b,lam", [(129, 2, 0.05), (192, 64, 0.5), (192, 64, 0.02), (256, 128, 0.3),
                                     (256, 100, 1.0), (200, 128, 1e-4)])
def test_score_bound_reduction_mixed_heads(n, b, lam, reps):
    # given scores whose spread differs per head: some heads keep few candidates under the bound
    # s_j >= s_(b) - lambda (finished by the reduced-footprint kernel), others keep nearly all
    # (handed on to the full-size kernel); quantised scores put ties on the bound itself.
    # reps = 23: 276 heads, more than one per CU, the batched kernels; reps = 1: a single small event
    h = 12 * reps
    K, V, _ = _mk(h, n, 7000 + n + b)
    g = torch.Generator().manual_seed(n * 131 + b)
    s = torch.randn((h, n), generator=g).exp()
    scale = torch.tensor([4.0, 1.0, 0.25, 0.05, 2.0, 1.0, 8.0, 0.5, 1.0, 3.0, 0.01, 1.5]).repeat(reps).view(h, 1)
    s = s * scale
    s[5::12] = torch.floor(s[5::12] * 4) / 4
    s[9::12] = torch.floor(s[9::12] * 2) / 2
    # near-duplicate value rows so that the penalty matters among the survivors
    V[:, n // 2:] = V[:, : n - n // 2] + 0.05 * V[:, n // 2:]
    s = s.to(DEV)
    data = {"K": K, "V": V, "s": s}
    out = B().kvr_retain(K, V, b, lam, 1e-6, s=s)
    torch.cuda.synchronize()
    heads = list(range(12)) + list(range(12, h, 11))
    rep = _check_heads(W.WORKLOADS["c3"], data, out, b, lam, 1e-6, heads)
    assert rep["heads"] == len(heads)
    sel = B().kvr_select_greedy(V, s, b, lam, 1e-6)
    torch.cuda.synchronize()
    assert torch.equal(sel[0], out.idx_sorted) and torch.equal(sel[1], out.pick_order)


@pytest.mark.parametrize("n,b,scale", [(300, 128, 1e-3), (1024, 128, 1e-3), (1024, 64, 1.0), (2048, 100, 1e-3),
                                       (2049, 128, 1e-3), (4096, 128, 1e-3), (4096, 30, 1.0), (700, 128, 0.05)])
def test_fp32_long_heads(n, b, scale):
    # fp32 rows of 257-4096 tokens with b <= 128 take the selection with lazily refreshed penalties on the fp32
    # MFMAs; scores far below lambda leave every token in play, near-duplicate rows make the penalty bite
    h = 3
    K, V, _ = _mk(h, n, 6100 + n + b, torch.float32)
    g = torch.Generator().manual_seed(n * 7 + b)
    s = (torch.randn((h, n), generator=g).exp() * scale).to(DEV)
    V[:, n // 2:] = V[:, : n - n // 2] + 0.05 * V[:, n // 2:]
    out = B().kvr_retain(K, V, b, 0.5, 1e-6, s=s)
    torch.cuda.synchronize()
    rep = _check_heads(W.WORKLOADS["c1"], {"K": K, "V": V, "s": s}, out, b, 0.5, 1e-6, range(h))
    assert rep["heads"] == h
    sel = B().kvr_select_greedy(V, s, b, 0.5, 1e-6)
    torch.cuda.synchronize()
    assert torch.equal(sel[0], out.idx_sorted) and torch.equal(sel[1], out.pick_order)


@pytest.mark.parametrize("n,b,lam", [(150, 16, 0.05), (192, 64, 0.5), (192, 64, 5.0), (256, 100, 0.3), (256, 128, 0.02),
                                     (129, 2, 0.5), (200, 128, 0.5)])
def test_fp32_rows_with_score_bound_reduction(n, b, lam):
    # fp32 heads of more than 128 tokens: with a small lambda (relative to the spread of the scores) the
    # kernel shrinks the head to the tokens the score bound leaves, with a large one it keeps all
    h = 6
    K, V, _ = _mk(h, n, 9900 + n + b, torch.float32)
    g = torch.Generator().manual_seed(n * 3 + b)
    s = torch.randn((h, n), generator=g).exp()
    s[1] = torch.floor(s[1] * 4) / 4                      # ties at the bound
    s[2, : n // 3] = 50.0                                 # a third of the tokens far above the rest
    s = s.to(DEV)
    V[:, n // 2:] = V[:, : n - n // 2] + 0.02 * V[:, n // 2:]
    out = B().kvr_retain(K, V, b, lam, 1e-6, s=s)
    torch.cuda.synchronize()
    _check_heads(W.WORKLOADS["c1"], {"K": K, "V": V, "s": s}, out, b, lam, 1e-6, range(h))


@pytest.mark.parametrize("n,b,G,lam", [(256, 128, 7, 0.5), (200, 64, 4, 0.3), (192, 150, 0, 0.5), (250, 40, 0, 0.0)])
def test_batched_and_single_event_kernels_agree_on_short_heads(n, b, G, lam):
    """Heads of 128 < n <= 256 tokens go through the sixteen-wave kernel when the call has at most one
    head per CU and through the four-wave kernel when it is batched: the same heads must give the
    same picks either way, and both are checked against the oracle."""
    h_big, h_small = 300, 40
    K, V, s = _mk(h_big, n, 7300 + n + b)
    V[:, n // 2:] = V[:, : n - n // 2] + 0.05 * V[:, n // 2:]
    g = torch.Generator().manual_seed(n + G)
    Q = torch.randn((h_big, G, 128), generator=g).to(torch.bfloat16).to(DEV) if G else None
    s = None if G else torch.randn((h_big, n), generator=g).exp().to(DEV)
    big = B().kvr_retain(K, V, b, lam, 1e-6, Q=Q, s=s)
    small = B().kvr_retain(K[:h_small].contiguous(), V[:h_small].contiguous(), b, lam, 1e-6,
                           Q=None if Q is None else Q[:h_small].contiguous(), s=None if s is None else s[:h_small].contiguous())
    torch.cuda.synchronize()
    assert torch.equal(big.pick_order[:h_small], small.pick_order)
    assert torch.equal(big.idx_sorted[:h_small], small.idx_sorted)
    assert torch.equal(big.K_out[:h_small], small.K_out) and torch.equal(big.V_out[:h_small], small.V_out)
    torch.testing.assert_close(big.pick_gain[:h_small], small.pick_gain, rtol=1e-5, atol=1e-7)
    data = {"K": K, "V": V}
    if G:
        data["Q"] = Q
    else:
        data["s"] = s
    _check_heads(W.WORKLOADS["c2"], data, big, b, lam, 1e-6, [0, 17, 150, 299])
    data_s = {k: v[:h_small] for k, v in data.items()}
    _check_heads(W.WORKLOADS["c2"], data_s, small, b, lam, 1e-6, [0, 17, 39])


@pytest.mark.parametrize("h,n,b,lam", [(4, 160, 70, 0.5), (3, 900, 100, 0.5), (2, 3000, 128, 0.25), (2, 5000, 60, 0.5)])
def test_exactly_representable_inputs_match_with_zero_near_ties(h, n, b, lam):
    # signed basis rows (norm 1, eps 0) with duplicates, dyadic scores and
    # lambda: every quantity is exact in fp32, so the picks must be the
    # oracle's, pick by pick (short heads, and the two long-head kernels)
    rng = np.random.default_rng(5)
    V = np.zeros((h, n, 128), dtype=np.float32)
    for hh in range(h):
        ax = rng.integers(0, 40, size=n)
        sg = rng.choice([-1.0, 1.0], size=n)
        V[hh, np.arange(n), ax] = sg
    s = (rng.permutation(h * n).reshape(h, n) / 16384.0).astype(np.float32)
    Vt = torch.tensor(V).to(torch.bfloat16).to(DEV)
    Kt = torch.tensor(rng.normal(size=(h, n, 128)).astype(np.float32)).to(torch.bfloat16).to(DEV)
    st = torch.tensor(s).to(DEV)
    out = B().kvr_retain(Kt, Vt, b, lam, 0.0, s=st)
    torch.cuda.synchronize()
    for hh in range(h):
        r = O.alpha_select(s[hh].astype(np.float64), V[hh].astype(np.float64), b, lam, 0.0)
        np.testing.assert_array_equal(out.pick_order[hh].cpu().numpy(), r["order"])
        np.testing.assert_array_equal(out.pick_gain[hh].cpu().numpy().astype(np.float64), r["gain"])
        np.testing.assert_array_equal(out.idx_sorted[hh].cpu().numpy(), r["sorted"])


@pytest.mark.parametrize("h,n,b", [(2, 130, 50), (2, 1000, 120), (1, 4000, 128), (1, 6000, 40)])
def test_identical_value_rows_and_score_ties(h, n, b):
    K, V, s = _mk(h, n, 3)
    V[:] = V[:, :1, :]
    s = torch.floor(s * 8) / 8                    # many exact ties
    out = B().kvr_retain(K, V, b, 0.75, 1e-6, s=s)
    torch.cuda.synchronize()
    data = {"K": K, "V": V, "s": s}
    _check_heads(W.WORKLOADS["c3"], data, out, b, 0.75, 1e-6, range(h))
    sn = s.cpu().numpy()
    for hh in range(h):
        want = np.argsort(-sn[hh], kind="stable")[:b]
        got = out.pick_order[hh].cpu().numpy()
        if n <= 256:
            np.testing.assert_array_equal(got, want)
        else:
            # long heads take the cosines of pool members and of refreshed tokens from two MFMA shapes, whose
            # fp32 sums may differ in the last bit: equal scores may swap (a near-tie for the oracle check
            # above), the score levels, an eighth apart, may not
            np.testing.assert_array_equal(sn[hh][got], sn[hh][want])


def test_lambda_zero_reads_no_values_and_is_stable_topb():
    h, n, b = 5, 500, 128
    K, V, s = _mk(h, n, 4)
    s = torch.floor(s * 64) / 64
    lay = B().layout_of(V)
    idx, order, gain = B().kvr_select_greedy(None, s, b, 0.0, lay=lay)
    torch.cuda.synchronize()
    sn = s.cpu().numpy()
    for hh in range(h):
        want = np.argsort(-sn[hh], kind="stable")[:b]
        np.testing.assert_array_equal(order[hh].cpu().numpy(), want)
        np.testing.assert_array_equal(idx[hh].cpu().numpy(), np.sort(want))
        np.testing.assert_array_equal(gain[hh].cpu().numpy(), sn[hh][want])


@pytest.mark.parametrize("n,b,dtype", [(257, 1, torch.bfloat16), (1000, 64, torch.bfloat16), (1024, 128, torch.bfloat16),
                                       (4096, 1024, torch.bfloat16), (5000, 300, torch.bfloat16), (8192, 1000, torch.bfloat16),
                                       (2048, 2047, torch.bfloat16), (700, 256, torch.float32), (3000, 17, torch.float32)])
@pytest.mark.parametrize("kind", ["wide", "quantised", "constant", "nonfinite"])
def test_lambda_zero_on_long_heads_is_the_stable_topb(n, b, dtype, kind):
    """Algorithm 1's explicit lambda = 0 branch on heads of more than 256 tokens: bit-exact top-b with
    ties to the lower index, whatever the scores hold, and the kept rows."""
    h = 4
    K, V, s = _mk(h, n, 4400 + n + b, dtype)
    if kind == "quantised":
        s = torch.floor(s * 8) / 8                         # many exact ties across the threshold
    elif kind == "constant":
        s = torch.zeros_like(s); s[1] = -0.0; s[2, ::3] = 1.0
    elif kind == "nonfinite":
        s[0, ::5] = float("inf"); s[1, 1::4] = float("-inf"); s[2, ::7] = float("nan"); s[3, :] = float("nan")
    out = B().kvr_retain(K, V, b, 0.0, 1e-6, s=s)
    torch.cuda.synchronize()
    sn = s.cpu().numpy()
    for hh in range(h):
        idx, order = out.idx_sorted[hh].cpu().numpy(), out.pick_order[hh].cpu().numpy()
        if kind == "nonfinite" and hh >= 2:                # NaN has no order: distinct, in range, rows kept
            assert len(set(idx.tolist())) == b and idx.min() >= 0 and idx.max() < n
            assert np.all(np.diff(idx) > 0) and sorted(order.tolist()) == idx.tolist()
        else:
            want = np.argsort(-(sn[hh] + 0.0), kind="stable")[:b]
            np.testing.assert_array_equal(order, want)
            np.testing.assert_array_equal(idx, np.sort(want))
            np.testing.assert_array_equal(out.pick_gain[hh].cpu().numpy(), sn[hh][want] + 0.0)
        np.testing.assert_array_equal(_bits(out.K_out[hh]), O.compact(_bits(K[hh]), idx))
        np.testing.assert_array_equal(_bits(out.V_out[hh]), O.compact(_bits(V[hh]), idx))


def test_strided_layout_and_separate_calls_equal_retain():
    h, n, b, G = 6, 200, 48, 3
    g = torch.Generator(device="cpu").manual_seed(9)
    big = torch.randn((h, n + 5, 136), generator=g).to(torch.bfloat16).to(DEV)
    bigv = torch.randn((h, n + 5, 136), generator=g).to(torch.bfloat16).to(DEV)
    K, V = big[:, :n, :128], bigv[:, :n, :128]
    Q = torch.randn((h, G, 128), generator=g).to(torch.bfloat16).to(DEV)
    out = B().kvr_retain(K, V, b, 0.5, 1e-6, Q=Q)
    s = B().kvr_score(K, Q)
    # the fused call may compute the logits on the matrix cores and the stand-alone
    # scorer with scalar FMAs: same scores up to fp32 rounding
    torch.testing.assert_close(s, out.s_out, rtol=2e-5, atol=0)
    idx, order, gain = B().kvr_select_greedy(V, out.s_out, b, 0.5, 1e-6)
    Ko, Vo = B().kvr_compact(K, V, idx)
    torch.cuda.synchronize()
    assert torch.equal(idx, out.idx_sorted)
    assert torch.equal(order, out.pick_order) and torch.equal(gain, out.pick_gain)
    assert torch.equal(Ko, out.K_out) and torch.equal(Vo, out.V_out)
    data = {"K": K.contiguous(), "V": V.contiguous(), "Q": Q}
    _check_heads(W.WORKLOADS["c2"], data, out, b, 0.5, 1e-6, range(h))


def test_compact_alone_and_idempotence():
    h, n, b = 3, 100, 20
    K, V, _ = _mk(h, n, 11)
    rng = np.random.default_rng(0)
    idx = np.stack([np.sort(rng.choice(n, b, replace=False)) for _ in range(h)]).astype(np.int32)
    it = torch.tensor(idx).to(DEV)
    Ko, Vo = B().kvr_compact(K, V, it)
    torch.cuda.synchronize()
    for hh in range(h):
        np.testing.assert_array_equal(_bits(Ko[hh]), O.compact(_bits(K[hh]), idx[hh]))
        np.testing.assert_array_equal(_bits(Vo[hh]), O.compact(_bits(V[hh]), idx[hh]))
    ident = torch.arange(b, dtype=torch.int32, device=DEV).repeat(h, 1)
    K2, _ = B().kvr_compact(Ko, None, ident)
    torch.cuda.synchronize()
    assert torch.equal(K2, Ko)


@pytest.mark.parametrize("name,heads,b,lam", [
    ("c1", 1, None, None), ("c2", 32, None, None), ("c3", 64, None, None), ("c3", 400, None, None),
    ("c5", 24, None, None), ("c5", 12, 64, 1.0), ("c5", 8, 200, None), ("c5", 8, None, 0.0), ("c4", 10, None, None)])
def test_runs_are_deterministic_and_stream_independent(name, heads, b, lam):
    # every kernel family: the same call three times, the third on another stream, bit for bit
    # (a race between waves or workgroups would show as a difference sooner or later)
    w = W.WORKLOADS[name]
    data = W.generate(w, heads=heads, seed=3, device=DEV)
    a, b, lam = _run(w, data, b=b, lam=lam)
    a2, _, _ = _run(w, data, b=b, lam=lam)
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        a3 = B().kvr_retain(data["K"], data["V"], b, lam, 1e-6, Q=data.get("Q"), s=data.get("s"), stream=st)
    st.synchronize()
    for other in (a2, a3):
        for f in ("idx_sorted", "pick_order", "pick_gain", "K_out", "V_out", "s_out"):
            x, y = getattr(a, f), getattr(other, f)
            if x is None and y is None:
                continue
            assert torch.equal(x, y), f


# ---------------------------------------------------------------- flat-signature mode
def _flat_case(seqs, group, n, seed, dtype):
    g = torch.Generator(device="cpu").manual_seed(seed)
    heads = seqs * group
    # heads of a sequence share a token geometry (cluster centres per token) plus head noise, so
    # that the mean over heads keeps a structure worth penalising
    base = torch.randn((seqs, 1, 12, 128), generator=g)[:, :, torch.randint(0, 12, (n,), generator=g)]
    V = (base + 0.5 * torch.randn((seqs, group, n, 128), generator=g)).reshape(heads, n, 128).to(dtype)
    K = torch.randn((heads, n, 128), generator=g).to(dtype)
    s = torch.randn((seqs, n), generator=g).exp()
    return K.to(DEV), V.to(DEV), s.to(DEV)


@pytest.mark.parametrize("seqs,group,n,b,lam,dtype", [
    (3, 8, 192, 64, 0.5, torch.bfloat16), (2, 32, 77, 30, 0.3, torch.bfloat16),
    (2, 5, 256, 128, 1.0, torch.bfloat16), (2, 4, 300, 40, 0.5, torch.bfloat16),
    (2, 6, 130, 20, 0.5, torch.float32), (2, 3, 64, 64, 0.0, torch.bfloat16),
    (1, 1, 4, 1, 0.2, torch.bfloat16), (4, 64, 10, 1, 0.2, torch.bfloat16), (2, 17, 500, 150, 0.5, torch.bfloat16),
    (2, 4, 1024, 128, 0.5, torch.bfloat16), (1, 3, 4096, 100, 0.5, torch.bfloat16), (2, 2, 2100, 128, 2.0, torch.bfloat16)])
def test_flat_signature_mode(seqs, group, n, b, lam, dtype):
    _flat_signature_mode(seqs, group, n, b, lam, dtype, 1.0)


@pytest.mark.parametrize("seqs,group,n,b", [(2, 4, 1024, 128), (1, 3, 4096, 128), (2, 2, 700, 64)])
def test_flat_signature_mode_with_scores_far_below_lambda(seqs, group, n, b):
    # long sequences whose scores the bound cannot thin out: every mean row is computed and every token stays in
    # play for the fp32 instance of the long-head kernel
    _flat_signature_mode(seqs, group, n, b, 0.5, torch.bfloat16, 1e-3)


def _flat_signature_mode(seqs, group, n, b, lam, dtype, score_scale):
    K, V, s = _flat_case(seqs, group, n, 9000 + n + group, dtype)
    s = (s * score_scale).contiguous()
    out = B().kvr_retain_flat(K, V, s, group, b, lam, 1e-6)
    torch.cuda.synchronize()
    V64 = W.to_f64(V).reshape(seqs, group, n, 128)
    Kb, Vb = _bits(K).reshape(seqs, group, n, -1), _bits(V).reshape(seqs, group, n, -1)
    for q in range(seqs):
        u64 = V64[q].mean(axis=0)
        s64 = W.to_f64(s[q])
        if lam != 0.0:
            # rows of tokens the score bound rules out (s_j < s_(b) - lambda) may be left zero; all others are the mean
            got = out.u_out[q].cpu().numpy()
            sure = s64 >= np.sort(s64)[::-1][b - 1] - lam
            tol = 2e-6 * np.abs(V64[q]).max()
            assert np.all(np.abs(got[sure] - u64[sure]) <= tol)
            rest = ~sure
            ok_rest = np.all(np.abs(got[rest] - u64[rest]) <= tol, axis=1) | np.all(got[rest] == 0.0, axis=1)
            assert np.all(ok_rest)
        idx = out.idx_sorted[q].cpu().numpy()
        P.check_head(s64, u64, b, lam, 1e-6, out.pick_order[q].cpu().numpy(), out.pick_gain[q].cpu().numpy(), idx)
        for g in range(group):
            h = q * group + g
            np.testing.assert_array_equal(_bits(out.K_out[h]), O.compact(Kb[q, g], idx))
            np.testing.assert_array_equal(_bits(out.V_out[h]), O.compact(Vb[q, g], idx))
    # the three steps called one by one give the same result
    if lam != 0.0:
        u = B().kvr_signature_flat(V, group)              # every row, also those the event leaves zero
        computed = out.u_out.abs().sum(dim=2) > 0
        assert torch.equal(u[computed], out.u_out[computed])
        lay = B().layout_of(u)
        sel = B().kvr_select_greedy(u, s, b, lam, 1e-6, lay=lay)
        assert torch.equal(sel[0], out.idx_sorted) and torch.equal(sel[1], out.pick_order)
    Ko, Vo = B().kvr_compact_shared(K, V, out.idx_sorted, group)
    torch.cuda.synchronize()
    assert torch.equal(Ko, out.K_out) and torch.equal(Vo, out.V_out)


@pytest.mark.parametrize("h", [6, 270])
@pytest.mark.parametrize("n,b,dtype", [(192, 64, torch.bfloat16), (100, 40, torch.bfloat16), (256, 128, torch.bfloat16),
                                       (150, 50, torch.float32)])
def test_non_finite_scores_still_give_distinct_indices_in_range(n, b, dtype, h):
    # unspecified picks, but never an index outside [0, n), never a duplicate, and finite heads
    # of the same launch are untouched (short heads only: these kernels run a fixed number of steps);
    # 6 heads: the single-event kernels, 270: the batched ones
    K, V, s = _mk(h, n, 4242 + n, dtype)
    s = s.clone()
    s[0, ::3] = float("nan")
    s[1, :] = float("-inf")
    s[2, 5] = float("inf"); s[2, 7] = float("inf")
    s[3, : n - b // 2] = float("nan")            # fewer finite scores than the budget
    V = V.clone()
    V[4, 3] = 0                                  # a zero row: zero signature, never penalised
    V[0, 10] = float("nan")                      # non-finite rows (in heads whose picks are unspecified anyway)
    V[2, 11, 5] = float("inf")
    out = B().kvr_retain(K, V, b, 0.5, 1e-6, s=s)
    torch.cuda.synchronize()
    idx = out.idx_sorted.cpu().numpy()
    order = out.pick_order.cpu().numpy()
    for hh in range(h):
        assert idx[hh].min() >= 0 and idx[hh].max() < n
        assert len(set(idx[hh].tolist())) == b and np.all(np.diff(idx[hh]) > 0)
        assert sorted(order[hh].tolist()) == idx[hh].tolist()
    data = {"K": K, "V": V, "s": s}
    _check_heads(W.WORKLOADS["c3"], data, out, b, 0.5, 1e-6, [4, 5, h - 1])
    assert order[2][0] == 5 and order[2][1] == 7          # +inf scores go first, lowest index first


@pytest.mark.parametrize("n,b,dtype", [(700, 64, torch.bfloat16), (1024, 128, torch.bfloat16), (3000, 100, torch.bfloat16),
                                       (5000, 64, torch.bfloat16), (1024, 200, torch.bfloat16), (900, 100, torch.float32)])
def test_non_finite_scores_on_long_heads_still_give_distinct_indices_in_range(n, b, dtype):
    # the same promise on the kernels for long heads, whose epochs are data-dependent: every loop ends (an epoch either
    # picks, or counts towards a limit after which the lowest unpicked tokens fill the list), the indices are distinct
    # and in range, and the finite heads of the launch are the oracle's
    h = 6
    K, V, s = _mk(h, n, 4343 + n, dtype)
    s = s.clone()
    s[0, ::3] = float("nan")
    s[1, :] = float("-inf")
    s[2, 5] = float("inf"); s[2, 7] = float("inf")
    s[3, : n - b // 2] = float("nan")            # fewer finite scores than the budget
    V = V.clone()
    V[4, 3] = 0                                  # a zero row: zero signature, never penalised
    V[0, 10] = float("nan")                      # non-finite rows (in heads whose picks are unspecified anyway)
    V[2, 11, 5] = float("inf")
    out = B().kvr_retain(K, V, b, 0.5, 1e-6, s=s)
    torch.cuda.synchronize()
    idx = out.idx_sorted.cpu().numpy()
    order = out.pick_order.cpu().numpy()
    for hh in range(h):
        assert idx[hh].min() >= 0 and idx[hh].max() < n
        assert len(set(idx[hh].tolist())) == b and np.all(np.diff(idx[hh]) > 0)
        assert sorted(order[hh].tolist()) == idx[hh].tolist()
    _check_heads(W.WORKLOADS["c3"], {"K": K, "V": V, "s": s}, out, b, 0.5, 1e-6, [4, 5])
    assert order[2][0] == 5 and order[2][1] == 7          # +inf scores go first, lowest index first


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_debug_validator_finds_non_finite_inputs(dtype):
    h, n, G = 5, 300, 3
    K, V, s = _mk(h, n, 515, dtype)
    Q = torch.randn((h, G, 128)).to(dtype).to(DEV)
    v = B().kvr_debug_validate_finite
    assert v(K=K, V=V, Q=Q, s=s)
    assert v(K=K) and v(V=V) and v(s=s, lay=B().layout_of(K)) and v(K=K, Q=Q)
    for which, plant in (("K", (4, 299, 127, float("nan"))), ("V", (0, 0, 0, float("inf"))),
                         ("V", (2, 150, 64, float("-inf"))), ("Q", (3, 2, 5, float("nan")))):
        t = {"K": K, "V": V, "Q": Q}[which].clone()
        t[plant[0], plant[1], plant[2]] = plant[3]
        args = {"K": K, "V": V, "Q": Q, "s": s}
        args[which] = t
        assert not v(**args), which
    for val in (float("nan"), float("inf"), float("-inf")):
        s2 = s.clone(); s2[h - 1, n - 1] = val
        assert not v(K=K, V=V, s=s2)
    # rows of a strided view: only the view's elements count
    big = torch.randn((h, n, 256)).to(dtype).to(DEV)
    big[:, :, 128:] = float("nan")
    assert v(K=big[:, :, :128])
    with pytest.raises(ValueError):
        v(K=big[:, :, :128], V=V)                        # one layout describes both: the strides must agree
    assert v(K=K, V=V, Q=Q, s=s)                         # the record is cleared by every call


def test_flat_mode_is_deterministic_and_group_one_is_the_per_head_selection():
    K, V, s = _flat_case(4, 1, 160, 77, torch.bfloat16)
    a = B().kvr_retain_flat(K, V, s, 1, 50, 0.5, 1e-6)
    c = B().kvr_retain_flat(K, V, s, 1, 50, 0.5, 1e-6)
    torch.cuda.synchronize()
    assert torch.equal(a.idx_sorted, c.idx_sorted) and torch.equal(a.pick_gain, c.pick_gain)
    computed = a.u_out.abs().sum(dim=2) > 0                 # (rows of tokens the score bound rules out stay zero)
    assert torch.equal(a.u_out[computed], V.float()[computed])   # the mean of one head is the head
    assert torch.equal(torch.gather(computed, 1, a.idx_sorted.long()), torch.ones_like(a.idx_sorted, dtype=torch.bool))
    data = {"K": K, "V": V, "s": s}
    per_head = B().kvr_retain(K, V, 50, 0.5, 1e-6, s=s)
    torch.cuda.synchronize()
    _check_heads(W.WORKLOADS["c3"], data, per_head, 50, 0.5, 1e-6, range(4))
    for q in range(4):
        P.check_head(W.to_f64(s[q]), W.to_f64(V[q]), 50, 0.5, 1e-6, a.pick_order[q].cpu().numpy(),
                     a.pick_gain[q].cpu().numpy(), a.idx_sorted[q].cpu().numpy())
    K2, V2, s2 = _flat_case(2, 16, 192, 78, torch.bfloat16)
    x = B().kvr_retain_flat(K2, V2, s2, 16, 64, 0.5, 1e-6)
    y = B().kvr_retain_flat(K2, V2, s2, 16, 64, 0.5, 1e-6)
    torch.cuda.synchronize()
    assert torch.equal(x.u_out, y.u_out) and torch.equal(x.pick_order, y.pick_order) and torch.equal(x.V_out, y.V_out)


def test_flat_mode_full_size_sampled_sequences():
    # c3's shape in the launch configuration bench.py --flat times: 32 sequences x 256 heads
    w = W.WORKLOADS["c3"]
    data = W.generate(w, seed=0, device=DEV)
    group = w.layers * w.kv_heads
    s = data["s"].view(w.seqs, group, w.n)[:, 0].contiguous()
    out = B().kvr_retain_flat(data["K"], data["V"], s, group, w.b, w.lam, 1e-6)
    torch.cuda.synchronize()
    for q in (0, 13, 31):
        sl = slice(q * group, (q + 1) * group)
        u64 = W.to_f64(data["V"][sl]).mean(axis=0)
        idx = out.idx_sorted[q].cpu().numpy()
        P.check_head(W.to_f64(s[q]), u64, w.b, w.lam, 1e-6, out.pick_order[q].cpu().numpy(),
                     out.pick_gain[q].cpu().numpy(), idx)
        for g in (0, 100, 255):
            h = q * group + g
            np.testing.assert_array_equal(_bits(out.K_out[h]), O.compact(_bits(data["K"][h]), idx))
            np.testing.assert_array_equal(_bits(out.V_out[h]), O.compact(_bits(data["V"][h]), idx))


def test_budgeted_frame_full_size_sampled_heads():
    # c3's shape in the launch configuration bench.py --budgeted times: 8192 heads, budgets in
    # [b/2, b], four sink tokens and a recent window of 16 protected, position ids
    w = W.WORKLOADS["c3"]
    data = W.generate(w, seed=0, device=DEV)
    g = torch.Generator(device=DEV).manual_seed(17)
    b_h = torch.randint(w.b // 2, w.b + 1, (w.heads,), generator=g, device=DEV, dtype=torch.int32)
    keep = torch.zeros((w.heads, w.n), dtype=torch.uint8, device=DEV)
    keep[:, :4] = 1
    keep[:, w.n - 16:] = 1
    pos = (torch.arange(w.n, dtype=torch.int32, device=DEV) * 2 + 1).repeat(w.heads, 1).contiguous()
    out = B().kvr_retain_budgeted(data["K"], data["V"], w.b, w.lam, 1e-6, s=data["s"], b_h=b_h, keep=keep, pos=pos)
    torch.cuda.synchronize()
    bh_all = b_h.cpu().numpy()
    idx_all = out.idx_sorted.cpu().numpy()
    # properties of every head: budget respected, ascending, protected tokens kept, padding
    valid = np.arange(w.b)[None, :] < bh_all[:, None]
    assert np.all(idx_all[~valid] == -1) and np.all(idx_all[valid] >= 0) and np.all(idx_all[valid] < w.n)
    assert np.all((np.diff(idx_all, axis=1) > 0) | ~valid[:, 1:])
    kept = np.zeros((w.heads, w.n), dtype=bool)
    rows = np.repeat(np.arange(w.heads), w.b).reshape(w.heads, w.b)
    kept[rows[valid], idx_all[valid]] = True
    assert kept[:, :4].all() and kept[:, w.n - 16:].all()
    kp = keep[0].cpu().numpy().astype(bool)
    for hh in np.random.default_rng(5).choice(w.heads, size=24, replace=False):
        bh = int(bh_all[hh])
        s64, V64 = W.to_f64(data["s"][hh]), W.to_f64(data["V"][hh])
        ref = O.select_budgeted(s64, V64, w.n, bh, kp, w.lam, 1e-6)
        order = out.pick_order[hh].cpu().numpy()
        gain = out.pick_gain[hh].cpu().numpy().astype(np.float64)
        idx = idx_all[hh]
        npz = len(ref["protected"])
        assert sorted(order[:npz].tolist()) == ref["protected"].tolist() and np.all(np.isinf(gain[:npz]))
        if order[npz:bh].tolist() == ref["order"].tolist():
            np.testing.assert_allclose(gain[npz:bh], ref["gain"], rtol=P.GAIN_RTOL,
                                       atol=P.GAIN_RTOL * (np.abs(s64).max() + w.lam))
        else:                                                    # a near-tie: every pick on the HIP path's own prefix
            Vh = O.signatures(V64, 1e-6); cos = Vh @ Vh.T
            S = list(order[:npz])
            for t in range(npz, bh):
                red = np.maximum(0.0, cos[:, S].max(axis=1))
                gt = s64 - w.lam * red
                gt[S] = -np.inf
                i = int(order[t])
                scale = max(abs(s64[i]) + w.lam * red[i], 1e-30)
                assert gt.max() - gt[i] <= P.NEAR_TIE * scale, (hh, t)
                assert abs(gain[t] - gt[i]) <= P.GAIN_RTOL * scale, (hh, t)
                S.append(i)
        assert sorted(order[:bh].tolist()) == idx[:bh].tolist()
        np.testing.assert_array_equal(_bits(out.K_out[hh])[:bh], O.compact(_bits(data["K"][hh]), idx[:bh]))
        np.testing.assert_array_equal(_bits(out.V_out[hh])[:bh], O.compact(_bits(data["V"][hh]), idx[:bh]))
        np.testing.assert_array_equal(out.pos_out[hh].cpu().numpy()[:bh], idx[:bh] * 2 + 1)


def test_observation_window_scores_full_size_sampled_heads():
    # c5 with an observation window of 32 positions (224 queries per head) and c4 with 64 (256):
    # the configurations bench.py --window times; scores of sampled heads against the oracle
    import dataclasses
    for name, window, sample in (("c5", 32, 6), ("c4", 64, 3)):
        w0 = W.WORKLOADS[name]
        w = dataclasses.replace(w0, G=w0.G * window)
        data = W.generate(w, seed=0, device=DEV)
        s = B().kvr_score(data["K"], data["Q"])
        torch.cuda.synchronize()
        assert torch.allclose(s.sum(dim=1), torch.ones(w.heads, device=DEV), atol=2e-4)
        for hh in np.random.default_rng(9).choice(w.heads, size=sample, replace=False):
            s64 = O.score_softmax_mean(W.to_f64(data["K"][hh]), W.to_f64(data["Q"][hh]))
            P.check_scores(s[hh].cpu().numpy(), s64)
        del data, s
        torch.cuda.empty_cache()


# ---------------------------------------------------------------- budgets and protected tokens
@pytest.mark.parametrize("n,b_max,lam,dtype,computed", [
    (192, 64, 0.5, torch.bfloat16, False), (256, 100, 0.3, torch.bfloat16, True), (120, 48, 0.7, torch.bfloat16, False),
    (600, 64, 0.5, torch.bfloat16, False), (150, 40, 0.5, torch.float32, False),
    # long heads with scores handed in: the kernel that shrinks them to their candidates takes the budgets too
    (1024, 128, 0.5, torch.bfloat16, False), (3000, 64, 0.5, torch.bfloat16, False), (2048, 100, 1.0, torch.bfloat16, False),
    (1024, 128, 0.5, torch.bfloat16, True)])
def test_budgeted_heads_and_protected_tokens(n, b_max, lam, dtype, computed):
    h = 8
    K, V, s = _mk(h, n, 5100 + n, dtype)
    g = torch.Generator().manual_seed(n)
    s = (torch.randn((h, n), generator=g).exp() * (0.02 if computed else 1.0)).to(DEV)
    V[:, n // 2:] = V[:, : n - n // 2] + 0.05 * V[:, n // 2:]      # near-duplicates: the penalty matters
    # head 2 has fewer candidates than b_max: the run for b_max runs dry, its budget does not
    n_h = torch.tensor([n, n - 7, b_max - 10, n, n, n - 1, b_max + 3, n], dtype=torch.int32)
    b_h = torch.tensor([b_max, b_max - 5, b_max // 2, 12, b_max, 9, b_max, 1], dtype=torch.int32)
    keep = torch.zeros((h, n), dtype=torch.uint8)
    keep[0, :4] = 1; keep[0, n - 8:] = 1                           # sinks and a recent window
    keep[1, :2] = 1
    keep[3, torch.randperm(n, generator=g)[:10]] = 1
    keep[5, n - 1 - 3: n - 1] = 1                                  # inside n_h = n - 1
    keep[7, 17] = 1                                                # budget 1, taken by the protected token
    pos = (torch.arange(n, dtype=torch.int32)[None, :] * 3 + torch.arange(h, dtype=torch.int32)[:, None]).contiguous()
    Q = torch.randn((h, 4, 128), generator=g).to(dtype).to(DEV) if computed else None
    out = B().kvr_retain_budgeted(K, V, b_max, lam, 1e-6, Q=Q, s=None if computed else s, n_h=n_h.to(DEV),
                                  b_h=b_h.to(DEV), keep=keep.to(DEV), pos=pos.to(DEV))
    torch.cuda.synchronize()
    Kb, Vb = _bits(K), _bits(V)
    for hh in range(h):
        nh, bh = int(n_h[hh]), int(b_h[hh])
        V64 = W.to_f64(V[hh])
        s64 = O.score_softmax_mean(W.to_f64(K[hh]), W.to_f64(Q[hh])) if computed else W.to_f64(s[hh])
        kp = keep[hh].numpy().astype(bool)
        ref = O.select_budgeted(s64, V64, nh, bh, kp, lam, 1e-6)
        order = out.pick_order[hh].cpu().numpy(); gain = out.pick_gain[hh].cpu().numpy().astype(np.float64)
        idx = out.idx_sorted[hh].cpu().numpy()
        npz = len(ref["protected"])
        assert np.all(order[bh:] == -1) and np.all(idx[bh:] == -1)
        assert sorted(order[:npz].tolist()) == ref["protected"].tolist() and np.all(np.isinf(gain[:npz]))
        assert sorted(order[:bh].tolist()) == idx[:bh].tolist() and idx[:bh].max() < nh
        # the greedy picks after the protected ones: every one must be the fp64 argmax of Eq. 2 on
        # the HIP path's own prefix, or within the near-tie bound of it
        Vh = O.signatures(V64[:nh], 1e-6); cos = Vh @ Vh.T
        S = list(order[:npz])
        for t in range(npz, bh):
            red = np.maximum(0.0, cos[:, S].max(axis=1)) if S else np.zeros(nh)
            gt = s64[:nh] - lam * red
            gt[S] = -np.inf
            i = int(order[t])
            scale = np.abs(s64[i]) + lam * red[i]
            assert gt.max() - gt[i] <= P.NEAR_TIE * max(scale, 1e-30), (hh, t)
            assert abs(gain[t] - gt[i]) <= P.GAIN_RTOL * max(scale, 1e-30), (hh, t)
            S.append(i)
        assert len(ref["order"]) == bh - npz
        np.testing.assert_array_equal(_bits(out.K_out[hh])[:bh], O.compact(Kb[hh], idx[:bh]))
        np.testing.assert_array_equal(_bits(out.V_out[hh])[:bh], O.compact(Vb[hh], idx[:bh]))
        assert not _bits(out.K_out[hh])[bh:].any()                 # rows past the budget are untouched (zeros)
        np.testing.assert_array_equal(out.pos_out[hh].cpu().numpy()[:bh], pos[hh].numpy()[idx[:bh]])
        assert np.all(out.pos_out[hh].cpu().numpy()[bh:] == -1)


@pytest.mark.parametrize("n,b_max,lam", [(192, 64, 0.5), (120, 48, 0.5), (256, 128, 0.3), (200, 32, 0.0),
                                         (600, 64, 0.5), (1024, 128, 0.5), (3000, 40, 1.0), (1000, 64, 0.0), (5000, 200, 0.0),
                                         (6000, 96, 0.5)])
def test_budgeted_heads_match_the_unbudgeted_prefix(n, b_max, lam):
    """On bf16 heads of up to 4096 tokens the fused kernels take the per-head budgets themselves.  The picks for
    budget b_h must be the first b_h picks of the plain run for b_max (a greedy pick depends on the
    earlier picks only), the kept rows the rows of exactly those picks, and a budget of zero
    writes nothing."""
    h = 24 if n <= 1024 else 8
    K, V, s = _mk(h, n, 6100 + n)
    g = torch.Generator().manual_seed(n + b_max)
    s = torch.randn((h, n), generator=g).exp().to(DEV)
    V[:, n // 2:] = V[:, : n - n // 2] + 0.05 * V[:, n // 2:]
    b_h = torch.randint(1, b_max + 1, (h,), generator=g, dtype=torch.int32)
    b_h[0], b_h[1], b_h[2], b_h[3] = b_max, 1, 0, 2
    full = B().kvr_retain(K, V, b_max, lam, 1e-6, s=s)
    out = B().kvr_retain_budgeted(K, V, b_max, lam, 1e-6, s=s, b_h=b_h.to(DEV))
    torch.cuda.synchronize()
    fo, fg = full.pick_order.cpu().numpy(), full.pick_gain.cpu().numpy()
    Kb, Vb = _bits(K), _bits(V)
    for hh in range(h):
        bh = int(b_h[hh])
        order, gain, idx = (out.pick_order[hh].cpu().numpy(), out.pick_gain[hh].cpu().numpy(),
                            out.idx_sorted[hh].cpu().numpy())
        np.testing.assert_array_equal(order[:bh], fo[hh][:bh])
        # (the two runs may take a head through different kernels, whose norms differ in the last bit)
        np.testing.assert_allclose(gain[:bh], fg[hh][:bh], rtol=1e-5)
        np.testing.assert_array_equal(idx[:bh], np.sort(fo[hh][:bh]))
        assert np.all(order[bh:] == -1) and np.all(idx[bh:] == -1) and np.all(np.isneginf(gain[bh:]))
        np.testing.assert_array_equal(_bits(out.K_out[hh])[:bh], O.compact(Kb[hh], idx[:bh]))
        np.testing.assert_array_equal(_bits(out.V_out[hh])[:bh], O.compact(Vb[hh], idx[:bh]))
        assert not _bits(out.K_out[hh])[bh:].any() and not _bits(out.V_out[hh])[bh:].any()
    # the plain run itself is checked against the oracle
    _check_heads(W.WORKLOADS["c3"], {"K": K, "V": V, "s": s}, full, b_max, lam, 1e-6, range(0, h, 5))


@pytest.mark.parametrize("n,b,dtype,G", [(8192, 24, torch.bfloat16, 0), (8192, 16, torch.float32, 256),
                                         (4096, 1024, torch.bfloat16, 0), (4096, 256, torch.bfloat16, 8),
                                         (256, 256, torch.bfloat16, 0), (192, 192, torch.float32, 0)])
def test_maximum_sizes(n, b, dtype, G):
    # the limits of the header (n = 8192, G = 256) and of the pool kernel (b = 1024)
    # kernels, and budgets that keep every token
    K, V, s = _mk(1, n, 8800 + n + b, dtype)
    g = torch.Generator().manual_seed(n + b)
    if G:
        Q = torch.randn((1, G, 128), generator=g).to(dtype).to(DEV)
        out = B().kvr_retain(K, V, b, 0.5, 1e-6, Q=Q)
        data = {"K": K, "V": V, "Q": Q}
    else:
        out = B().kvr_retain(K, V, b, 0.5, 1e-6, s=s)
        data = {"K": K, "V": V, "s": s}
    torch.cuda.synchronize()
    rep = _check_heads(W.WORKLOADS["c3"], data, out, b, 0.5, 1e-6, [0])
    assert rep["heads"] == 1
    if b == n:
        assert out.idx_sorted[0].cpu().tolist() == list(range(n))


@pytest.mark.parametrize("n,b_max", [(192, 64), (600, 48)])
def test_budgeted_per_head_lambda(n, b_max):
    # head h runs with lambda_h[h]: the kernels see scores scaled by lambda/lambda_h and the one
    # launch lambda, the gains come back on the head's own scale
    h = 6
    K, V, s = _mk(h, n, 6100 + n)
    V[:, n // 2:] = V[:, : n - n // 2] + 0.05 * V[:, n // 2:]
    lam_h = torch.tensor([0.05, 0.25, 0.5, 1.0, 2.0, 0.5], dtype=torch.float32)
    b_h = torch.tensor([b_max, b_max, b_max - 3, b_max, 7, b_max], dtype=torch.int32)
    out = B().kvr_retain_budgeted(K, V, b_max, 0.5, 1e-6, s=s, b_h=b_h.to(DEV), lam_h=lam_h.to(DEV))
    torch.cuda.synchronize()
    for hh in range(h):
        bh, lam = int(b_h[hh]), float(lam_h[hh])
        P.check_head(W.to_f64(s[hh]), W.to_f64(V[hh]), bh, lam, 1e-6, out.pick_order[hh].cpu().numpy()[:bh],
                     out.pick_gain[hh].cpu().numpy()[:bh], out.idx_sorted[hh].cpu().numpy()[:bh])
    # heads 2 and 5 share lambda = the launch lambda: their scores went through unscaled
    same = B().kvr_retain(K[5:6].contiguous(), V[5:6].contiguous(), b_max, 0.5, 1e-6, s=s[5:6].contiguous())
    torch.cuda.synchronize()
    # (another kernel may serve the plain call: the same picks, gains to fp32 rounding of a different summation order)
    assert torch.equal(same.pick_order[0], out.pick_order[5])
    torch.testing.assert_close(same.pick_gain[0], out.pick_gain[5], rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("n,dtype", [(200, torch.bfloat16), (150, torch.float32), (700, torch.bfloat16), (5000, torch.bfloat16)])
def test_strided_layouts_in_every_mode(n, dtype):
    # K and V are views into larger buffers (token stride 136, extra tokens per head): the
    # strided calls must give what the same calls give on contiguous copies
    h, b, group = 6, 40, 3
    g = torch.Generator(device="cpu").manual_seed(19 + n)
    bigk = torch.randn((h, n + 5, 136), generator=g).to(dtype).to(DEV)
    bigv = torch.randn((h, n + 5, 136), generator=g).to(dtype).to(DEV)
    K, V = bigk[:, :n, :128], bigv[:, :n, :128]
    Kc, Vc = K.contiguous(), V.contiguous()
    s = torch.randn((h, n), generator=g).exp().to(DEV)
    a, c = B().kvr_retain(K, V, b, 0.5, 1e-6, s=s), B().kvr_retain(Kc, Vc, b, 0.5, 1e-6, s=s)
    torch.cuda.synchronize()
    assert torch.equal(a.pick_order, c.pick_order) and torch.equal(a.K_out, c.K_out) and torch.equal(a.V_out, c.V_out)
    _check_heads(W.WORKLOADS["c3"], {"K": Kc, "V": Vc, "s": s}, a, b, 0.5, 1e-6, range(h))
    sf = s[: h // group].contiguous()
    a, c = B().kvr_retain_flat(K, V, sf, group, b, 0.5, 1e-6), B().kvr_retain_flat(Kc, Vc, sf, group, b, 0.5, 1e-6)
    torch.cuda.synchronize()
    assert torch.equal(a.u_out, c.u_out) and torch.equal(a.pick_order, c.pick_order)
    assert torch.equal(a.K_out, c.K_out) and torch.equal(a.V_out, c.V_out)
    b_h = torch.tensor([b, b - 3, 5, b, 1, b // 2], dtype=torch.int32, device=DEV)
    keep = torch.zeros((h, n), dtype=torch.uint8, device=DEV)
    keep[:, :2] = 1
    a = B().kvr_retain_budgeted(K, V, b, 0.5, 1e-6, s=s, b_h=b_h, keep=keep)
    c = B().kvr_retain_budgeted(Kc, Vc, b, 0.5, 1e-6, s=s, b_h=b_h, keep=keep)
    torch.cuda.synchronize()
    assert torch.equal(a.idx_sorted, c.idx_sorted) and torch.equal(a.K_out, c.K_out) and torch.equal(a.V_out, c.V_out)
    # lambda = 0 (the top-b kernel on long heads), plain and with budgets
    a, c = B().kvr_retain(K, V, b, 0.0, 1e-6, s=s), B().kvr_retain(Kc, Vc, b, 0.0, 1e-6, s=s)
    torch.cuda.synchronize()
    assert torch.equal(a.pick_order, c.pick_order) and torch.equal(a.K_out, c.K_out) and torch.equal(a.V_out, c.V_out)
    _check_heads(W.WORKLOADS["c3"], {"K": Kc, "V": Vc, "s": s}, a, b, 0.0, 1e-6, range(h))
    a = B().kvr_retain_budgeted(K, V, b, 0.0, 1e-6, s=s, b_h=b_h, keep=keep)
    c = B().kvr_retain_budgeted(Kc, Vc, b, 0.0, 1e-6, s=s, b_h=b_h, keep=keep)
    torch.cuda.synchronize()
    assert torch.equal(a.idx_sorted, c.idx_sorted) and torch.equal(a.K_out, c.K_out) and torch.equal(a.V_out, c.V_out)


@pytest.mark.parametrize("n,G", [(200, 12), (256, 32), (900, 28), (984, 32), (1500, 20)])
def test_scores_from_a_wide_query_window(n, G):
    # G up to 32 queries per head (an observation window of several steps times the grouped
    # queries) go through the matrix-core scorer as long as the logits fit the LDS
    h, b = 3, 40
    K, V, _ = _mk(h, n, 7700 + n + G)
    g = torch.Generator().manual_seed(G * 1000 + n)
    Q = torch.randn((h, G, 128), generator=g).to(torch.bfloat16).to(DEV)
    out = B().kvr_retain(K, V, b, 0.5, 1e-6, Q=Q)
    s = B().kvr_score(K, Q)
    torch.cuda.synchronize()
    torch.testing.assert_close(s, out.s_out, rtol=2e-5, atol=0)
    _check_heads(W.WORKLOADS["c2"], {"K": K, "V": V, "Q": Q}, out, b, 0.5, 1e-6, range(h))


@pytest.mark.parametrize("n,G,sharp,strided", [
    (1, 40, 1.0, False), (33, 200, 1.0, False), (1000, 33, 1.0, False), (1500, 20, 4.0, False),
    (4096, 8, 1.0, False), (777, 100, 2.0, True), (4096, 256, 1.0, False), (8192, 64, 1.0, False),
    (2050, 255, 6.0, False),
    # the LDS-resident scorer with eight waves per workgroup (large logit buffers), ragged last tiles
    (3001, 8, 1.0, False), (899, 32, 2.0, False), (2047, 5, 1.0, True)])
def test_scores_from_an_observation_window_of_up_to_256_queries(n, G, sharp, strided):
    """W recent positions x grouped heads as one wide Q: the two-pass matrix-core scorer (any n, G <= 256).
    `sharp` scales the queries: peaked softmaxes, logits tens of units apart."""
    h = 3
    g = torch.Generator().manual_seed(G * 10000 + n)
    if strided:
        Kbuf = torch.randn((h, n + 5, 192), generator=g).to(torch.bfloat16).to(DEV)
        K = Kbuf[:, :n, 32:160]
    else:
        K = torch.randn((h, n, 128), generator=g).to(torch.bfloat16).to(DEV)
    Q = (torch.randn((h, G, 128), generator=g) * sharp).to(torch.bfloat16).to(DEV)
    Q[1, G // 2] = 0                                   # a query with a flat softmax
    s = B().kvr_score(K, Q)
    torch.cuda.synchronize()
    for hh in range(h):
        s64 = O.score_softmax_mean(W.to_f64(K[hh]), W.to_f64(Q[hh]))
        P.check_scores(s[hh].cpu().numpy(), s64)
        assert abs(float(s[hh].sum()) - 1.0) < 1e-4    # a mean of softmaxes sums to one
    # the whole event on these scores
    if n >= 64:
        V = torch.randn((h, n, 128), generator=g).to(torch.bfloat16).to(DEV)
        out = B().kvr_retain(K.contiguous(), V, 24, 0.5, 1e-6, Q=Q)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(out.s_out.cpu().numpy(), s.cpu().numpy())
        _check_heads(W.WORKLOADS["c2"], {"K": K.contiguous(), "V": V, "Q": Q}, out, 24, 0.5, 1e-6, range(h))


@pytest.mark.parametrize("n,kernel", [(1, 7), (6, 3), (192, 7), (1000, 13), (4096, 5), (300, 63), (257, 1)])
def test_score_pooling(n, kernel):
    heads = 7
    g = torch.Generator().manual_seed(n + kernel)
    s = torch.randn((heads, n), generator=g).exp().to(DEV)
    mx = B().kvr_score_pool(s, kernel, B().KVR_POOL_MAX)
    mean = B().kvr_score_pool(s, kernel, B().KVR_POOL_MEAN)
    torch.cuda.synchronize()
    for h in range(heads):
        s64 = W.to_f64(s[h])
        np.testing.assert_array_equal(mx[h].cpu().numpy().astype(np.float64), O.score_pool(s64, kernel))
        want = O.score_pool(s64, kernel, mean=True)
        got = mean[h].cpu().numpy().astype(np.float64)
        scale = O.score_pool(np.abs(s64), kernel, mean=True)
        assert np.all(np.abs(got - want) <= 1e-5 * scale)
    # pooled scores feed the selection like any others
    if n >= 6:
        V = torch.randn((heads, n, 128), generator=g).to(torch.bfloat16).to(DEV)
        b = max(1, n // 4)
        idx, order, gain = B().kvr_select_greedy(V, mx, b, 0.5)
        torch.cuda.synchronize()
        for h in (0, heads - 1):
            P.check_head(W.to_f64(mx[h]), W.to_f64(V[h]), b, 0.5, 1e-6, order[h].cpu().numpy(),
                         gain[h].cpu().numpy(), idx[h].cpu().numpy())


def _random_index_rows(rows, n, b, seed, kind):
    """Strictly ascending index rows of the kinds an eviction step produces, -1 padded."""
    rng = np.random.default_rng(seed)
    idx = np.full((rows, b), -1, dtype=np.int32)
    for r in range(rows):
        if kind == "shift":                   # every destination is the source of the row before it
            m = min(b, n - 1)
            idx[r, :m] = np.arange(1, m + 1)
        elif kind == "identity_prefix":       # a kept prefix (sinks), then a sparse tail
            keep = b // 2
            idx[r, :keep] = np.arange(keep)
            idx[r, keep:] = keep + np.sort(rng.choice(n - keep, size=b - keep, replace=False))
        elif kind == "ragged":                # per-head budgets: a valid prefix, then padding
            m = int(rng.integers(0, b + 1))
            idx[r, :m] = np.sort(rng.choice(n, size=m, replace=False))
        else:
            idx[r] = np.sort(rng.choice(n, size=b, replace=False))
    return idx


@pytest.mark.parametrize("kind", ["random", "shift", "identity_prefix", "ragged"])
@pytest.mark.parametrize("n,b,dtype,strided", [
    (192, 64, torch.bfloat16, False), (1, 1, torch.bfloat16, False), (100, 100, torch.float32, False),
    (777, 300, torch.bfloat16, True), (4096, 4095, torch.bfloat16, False), (1500, 257, torch.float32, True),
    (8192, 4100, torch.bfloat16, False)])
def test_inplace_compaction(kind, n, b, dtype, strided):
    heads = 6 if n <= 4096 else 2
    g = torch.Generator().manual_seed(n * 7 + b)
    if strided:     # rows padded to 160 elements, heads padded by 3 rows
        Kbuf = torch.randn((heads, n + 3, 160), generator=g).to(dtype).to(DEV)
        Vbuf = torch.randn((heads, n + 3, 160), generator=g).to(dtype).to(DEV)
        K, V = Kbuf[:, :n, :128], Vbuf[:, :n, :128]
    else:
        Kbuf = torch.randn((heads, n, 128), generator=g).to(dtype).to(DEV)
        Vbuf = torch.randn((heads, n, 128), generator=g).to(dtype).to(DEV)
        K, V = Kbuf, Vbuf
    K0, V0, Kbuf0 = _bits(K), _bits(V), _bits(Kbuf)
    idx = _random_index_rows(heads, n, b, n + b, kind)
    pos0 = (np.arange(n, dtype=np.int32)[None, :] * 5 + np.arange(heads, dtype=np.int32)[:, None] * 100003)
    pos = torch.from_numpy(pos0.copy()).to(DEV)
    B().kvr_compact_inplace(K, V, torch.from_numpy(idx).to(DEV), pos=pos)
    torch.cuda.synchronize()
    K1, V1, p1 = _bits(K), _bits(V), pos.cpu().numpy()
    for h in range(heads):
        np.testing.assert_array_equal(K1[h], O.compact_inplace(K0[h], idx[h]))
        np.testing.assert_array_equal(V1[h], O.compact_inplace(V0[h], idx[h]))
        np.testing.assert_array_equal(p1[h], O.compact_inplace(pos0[h], idx[h]))
    if strided:     # the padding between rows and heads is not written
        Kb1 = _bits(Kbuf)
        np.testing.assert_array_equal(Kb1[:, :, 128:], Kbuf0[:, :, 128:])
        np.testing.assert_array_equal(Kb1[:, n:], Kbuf0[:, n:])


def test_inplace_compaction_after_a_budgeted_selection_and_with_a_shared_list():
    """The eviction step as a serving loop runs it: select without output rows, then move the
    rows inside the cache; and flat mode, where the heads of a sequence share one index row."""
    h, n, b_max = 8, 192, 64
    K, V, s = _mk(h, n, 9100)
    b_h = torch.tensor([64, 10, 1, 33, 64, 5, 64, 17], dtype=torch.int32)
    pos = torch.arange(n, dtype=torch.int32).repeat(h, 1).contiguous().to(DEV)
    out = B().kvr_retain_budgeted(K, V, b_max, 0.5, 1e-6, s=s, b_h=b_h.to(DEV), pos=pos)
    torch.cuda.synchronize()
    Kc, Vc, pc = K.clone(), V.clone(), pos.clone()
    B().kvr_compact_inplace(Kc, Vc, out.idx_sorted, pos=pc)
    torch.cuda.synchronize()
    for hh in range(h):
        bh = int(b_h[hh])
        np.testing.assert_array_equal(_bits(Kc[hh])[:bh], _bits(out.K_out[hh])[:bh])      # same rows as the
        np.testing.assert_array_equal(_bits(Vc[hh])[:bh], _bits(out.V_out[hh])[:bh])      # out-of-place call
        np.testing.assert_array_equal(_bits(Kc[hh])[bh:], _bits(K[hh])[bh:])
        np.testing.assert_array_equal(pc[hh].cpu().numpy()[:bh], out.pos_out[hh].cpu().numpy()[:bh])
    # shared list: 3 sequences of 4 heads
    K, V, _ = _mk(12, 300, 9200)
    idx = _random_index_rows(3, 300, 77, 4, "random")
    K0, V0 = _bits(K), _bits(V)
    B().kvr_compact_inplace(K, None, torch.from_numpy(idx).to(DEV), group=4)      # K only
    torch.cuda.synchronize()
    for hh in range(12):
        np.testing.assert_array_equal(_bits(K[hh]), O.compact_inplace(K0[hh], idx[hh // 4]))
    np.testing.assert_array_equal(_bits(V), V0)


@pytest.mark.parametrize("n,dtype,strided", [(1, torch.bfloat16, False), (17, torch.float32, False), (300, torch.float32, False), (256, torch.bfloat16, True), (1024, torch.bfloat16, False),
                                             (192, torch.bfloat16, False), (777, torch.bfloat16, True),
                                             (1500, torch.float32, True), (4096, torch.bfloat16, False),
                                             (8192, torch.bfloat16, False)])
def test_mean_direction_prior_scores(n, dtype, strided):
    """The rejected modular variant: s + lambda_p cos(V_i, mean row).  Scores to the 1e-4 bar, on
    the scale |s| + |lambda_p|; top-b of them is then the ordinary lambda = 0 path."""
    heads = 5
    g = torch.Generator().manual_seed(n)
    if strided:
        Vbuf = torch.randn((heads, n + 2, 136), generator=g).to(dtype).to(DEV)
        V = Vbuf[:, :n, :128]
    else:
        V = torch.randn((heads, n, 128), generator=g).to(dtype).to(DEV)
    V[1] = V[1] + 2.0                       # a head with a strong common direction
    m = V[2, 1::2].shape[0]
    if m:
        V[2, 1::2] = -V[2, 0:2 * m:2]       # rows cancelling in pairs: dir is 0 (n even) or one row / n
    V[3] = 0                                # all-zero head: dir = 0, every cosine 0
    s = torch.randn((heads, n), generator=g).to(DEV)
    for lam_p in (0.5, -1.25):
        out = B().kvr_score_prior(V, s, lam_p, 1e-6)
        torch.cuda.synchronize()
        for h in range(heads):
            want = O.score_mean_direction_prior(W.to_f64(s[h]), W.to_f64(V[h]), lam_p, 1e-6)
            got = out[h].cpu().numpy().astype(np.float64)
            scale = np.abs(W.to_f64(s[h])) + abs(lam_p)
            assert np.all(np.abs(got - want) <= P.GAIN_RTOL * scale), (h, np.abs(got - want).max())
        np.testing.assert_array_equal(out[3].cpu().numpy(), s[3].cpu().numpy())
    # in place, and as the input of the lambda = 0 selection
    s2 = s.clone()
    B().kvr_score_prior(V, s2, 0.5, 1e-6, s_out=s2)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(s2.cpu().numpy(), B().kvr_score_prior(V, s, 0.5, 1e-6).cpu().numpy())
    b = max(1, n // 3)
    _, order, _ = B().kvr_select_greedy(V, s2, b, 0.0)
    torch.cuda.synchronize()
    for h in range(heads):
        want = O.topk_order(s2[h].cpu().numpy().astype(np.float64), b)
        np.testing.assert_array_equal(order[h].cpu().numpy(), want)


@pytest.mark.parametrize("seed", [1, 2, 3, 4, 5])
def test_seeded_sweep_over_shapes_dtypes_and_score_kinds(seed):
    # forty seeded cases per seed across every kernel the dispatch can choose (a few heads or hundreds): head lengths 1..8192,
    # budgets 1..n, lambda in {0, .05, .5, 1, 3}, bf16 and fp32 rows, given scores of wide and tight
    # spread (quantised now and then, so that ties occur), computed scores from 1..256 queries
    rng = np.random.default_rng(seed)
    for case in range(40):
        dtype = torch.bfloat16 if rng.random() < 0.8 else torch.float32
        nmax = 8192 if dtype == torch.bfloat16 else 600
        n = int(rng.choice([rng.integers(1, 70), rng.integers(64, 260), rng.integers(257, nmax)]))
        b = int(rng.integers(1, min(n, 300) + 1))
        if rng.random() < 0.3:
            b = min(n, int(rng.choice([1, 2, 64, 128, 700, n])))
        if n > 4096:
            b = min(b, 1024)                           # (beyond that: one pass over V per pick, seconds per head)
        lam = float(rng.choice([0.0, 0.05, 0.5, 1.0, 3.0]))
        h = int(rng.integers(1, 4))
        if n <= 256 and rng.random() < 0.25:
            h = int(rng.integers(257, 500))            # more heads than CUs: the batched kernels
        kind = rng.choice(["given_wide", "given_tight", "computed"])
        g = torch.Generator().manual_seed(int(rng.integers(1 << 30)))
        K = torch.randn((h, n, 128), generator=g).to(dtype).to(DEV)
        V = torch.randn((h, n, 128), generator=g).to(dtype)
        if rng.random() < 0.5 and n > 4:
            V[:, n // 2:] = V[:, : n - n // 2] + 0.05 * V[:, n // 2:]
        V = V.to(DEV)
        data = {"K": K, "V": V}
        if kind == "computed":
            G = int(rng.choice([1, 4, 7, 8, 12, 32, 33, 100, 256]))
            data["Q"] = torch.randn((h, G, 128), generator=g).to(dtype).to(DEV)
        else:
            s = torch.randn((h, n), generator=g).exp() * (1.0 if kind == "given_wide" else 0.01)
            if rng.random() < 0.2:
                s = torch.floor(s * 4) / 4
            data["s"] = s.to(DEV)
        out = B().kvr_retain(K, V, b, lam, 1e-6, Q=data.get("Q"), s=data.get("s"))
        torch.cuda.synchronize()
        check = range(h) if h <= 3 else sorted(set([0, h - 1] + rng.choice(h, size=2, replace=False).tolist()))
        try:
            _check_heads(W.WORKLOADS["c3"], data, out, b, lam, 1e-6, check)
        except AssertionError as e:
            raise AssertionError(f"case {case}: n={n} b={b} lambda={lam} heads={h} {kind} {dtype}: {e}") from e



@pytest.mark.parametrize("n,b", [(192, 64), (600, 48), (1024, 64), (3000, 40), (1024, 300), (5000, 24), (8000, 100)])
def test_gains_within_one_percent_of_each_other(n, b):
    """Every gain of the event lies in [1.5014, 1.507): values that agree in their sign, exponent
    and leading seven mantissa bits, so a candidate choice that looks at those bits only cannot
    tell the tokens apart and has to fall back on the full values."""
    heads = 3
    g = torch.Generator(device="cpu").manual_seed(4200 + n)
    K = torch.randn((heads, n, 128), generator=g).to(torch.bfloat16)
    V = torch.randn((heads, n, 128), generator=g).to(torch.bfloat16)
    s = (1.502 + 0.005 * torch.rand((heads, n), generator=g)).to(torch.float32)
    lam = 0.002
    data = {"K": K.to(DEV), "V": V.to(DEV), "s": s.to(DEV)}
    out = B().kvr_retain(data["K"], data["V"], b, lam, 1e-6, s=data["s"])
    torch.cuda.synchronize()
    rep = _check_heads(W.WORKLOADS["c5"], data, out, b, lam, 1e-6, range(heads))
    print(f"\n[crowded gains n={n}] {rep}")
    assert rep["heads"] == heads


def _adversarial_scores(kind, heads, n, g):
    u = torch.rand((heads, n), generator=g)
    if kind == "crowded":                      # one 16-bit key bucket
        return 1.502 + 0.005 * u
    if kind == "negative_crowded":
        return -1.507 + 0.005 * u
    if kind == "huge_range":                   # 60 decades
        return torch.pow(10.0, 60.0 * u - 30.0)
    if kind == "signed":
        return torch.randn((heads, n), generator=g)
    raise ValueError(kind)


def _adversarial_rows(kind, heads, n, g):
    V = torch.randn((heads, n, 128), generator=g)
    if kind == "zero_rows":                    # v = 0/(0 + eps) = 0: cosine 0 to everything
        V[:, ::5] = 0.0
    elif kind == "norms_near_eps":             # ||V_i|| between 0.3 eps and 30 eps: the + eps of Eq. 1 decides the cosines
        V = V * (1e-6 / 11.3) * torch.pow(10.0, 2.0 * torch.rand((heads, n, 1), generator=g) - 0.5)
    elif kind == "duplicates":                 # every row occurs four times
        V = V[:, : (n + 3) // 4].repeat(1, 4, 1)[:, :n]
        V = V[:, torch.randperm(n, generator=g)]
    elif kind == "scaled":                     # norms over six decades, directions in a few clusters
        c = torch.randn((heads, 12, 128), generator=g)
        V = c[:, torch.randint(0, 12, (n,), generator=g)] + 0.1 * V
        V = V * torch.pow(10.0, 6.0 * torch.rand((heads, n, 1), generator=g) - 3.0)
    else:
        raise ValueError(kind)
    return V


@pytest.mark.parametrize("rows", ["scaled", "duplicates", "zero_rows"])
@pytest.mark.parametrize("scores", ["crowded", "negative_crowded"])
@pytest.mark.parametrize("n,b,lam,dtype", [(1069, 128, 3.0, torch.bfloat16), (527, 128, 1.0, torch.float32),
                                           (3000, 128, 1.0, torch.bfloat16), (4096, 100, 3.0, torch.float32),
                                           (700, 64, 0.5, torch.bfloat16), (6000, 128, 3.0, torch.bfloat16),
                                           (1024, 200, 1.0, torch.bfloat16)])
def test_crowded_scores_under_a_large_lambda(n, b, lam, dtype, scores, rows):
    """Scores within a hair of each other and a penalty that dwarfs their spread: after the first picks most
    tokens carry the same out-of-date bound, far above every up-to-date gain.  The selection with lazily
    refreshed penalties has to bring that whole crowd up to date before it can go on (it once refreshed it
    a token at a time and gave up); the kernels that pass over all of V per epoch are run on the same inputs."""
    heads = 2
    g = torch.Generator(device="cpu").manual_seed(9100 + 7 * n + 31 * len(scores) + 101 * len(rows))
    K = torch.randn((heads, n, 128), generator=g).to(dtype)
    V = _adversarial_rows(rows, heads, n, g).to(dtype)
    s = _adversarial_scores(scores, heads, n, g).to(torch.float32)
    data = {"K": K.to(DEV), "V": V.to(DEV), "s": s.to(DEV)}
    out = B().kvr_retain(data["K"], data["V"], b, lam, 1e-6, s=data["s"])
    torch.cuda.synchronize()
    assert torch.isfinite(out.pick_gain).all()                 # (a head that gives up logs -inf gains)
    rep = _check_heads(W.WORKLOADS["c3" if dtype == torch.bfloat16 else "c1"], data, out, b, lam, 1e-6, range(heads))
    assert rep["heads"] == heads


@pytest.mark.parametrize("rows", ["zero_rows", "norms_near_eps", "duplicates", "scaled"])
@pytest.mark.parametrize("scores", ["crowded", "negative_crowded", "huge_range", "signed"])
@pytest.mark.parametrize("n,b,heads,dtype", [(100, 40, 300, torch.bfloat16), (192, 64, 300, torch.bfloat16),
                                             (256, 128, 2, torch.bfloat16), (700, 64, 2, torch.bfloat16),
                                             (2500, 48, 1, torch.bfloat16), (150, 50, 2, torch.float32)])
def test_adversarial_scores_and_rows(n, b, heads, dtype, scores, rows):
    """Score distributions and value rows chosen against the kernels' shortcuts (cut keys, score
    bounds, norms): every kernel the dispatch picks for these shapes, a few heads checked each."""
    g = torch.Generator(device="cpu").manual_seed(7000 + 13 * n + 101 * len(scores) + 1009 * len(rows))
    K = torch.randn((heads, n, 128), generator=g).to(dtype)
    V = _adversarial_rows(rows, heads, n, g).to(dtype)
    s = _adversarial_scores(scores, heads, n, g).to(torch.float32)
    lam = {"crowded": 0.002, "negative_crowded": 0.002, "huge_range": 0.5, "signed": 0.7}[scores]
    data = {"K": K.to(DEV), "V": V.to(DEV), "s": s.to(DEV)}
    out = B().kvr_retain(data["K"], data["V"], b, lam, 1e-6, s=data["s"])
    torch.cuda.synchronize()
    check = sorted(set([0, 1 % heads, heads // 2, heads - 1]))
    rep = _check_heads(W.WORKLOADS["c3"], data, out, b, lam, 1e-6, check)
    assert rep["heads"] == len(check)


def _check_budgeted_head(out, hh, K, V, s64, nh, bh, kp, lam, pos):
    """One head of a budgeted call against the oracle: protected tokens first, then Eq. 2-3 on the
    HIP path's own prefix, padding, kept rows and position ids."""
    V64 = W.to_f64(V[hh])
    ref = O.select_budgeted(s64, V64, nh, bh, kp, lam, 1e-6)
    order = out.pick_order[hh].cpu().numpy(); gain = out.pick_gain[hh].cpu().numpy().astype(np.float64)
    idx = out.idx_sorted[hh].cpu().numpy()
    npz = len(ref["protected"])
    assert np.all(order[bh:] == -1) and np.all(idx[bh:] == -1)
    assert sorted(order[:npz].tolist()) == ref["protected"].tolist() and np.all(np.isinf(gain[:npz]))
    assert sorted(order[:bh].tolist()) == idx[:bh].tolist()
    if bh:
        assert idx[:bh].max() < nh and len(set(idx[:bh].tolist())) == bh
    Vh = O.signatures(V64[:nh], 1e-6); cos = Vh @ Vh.T
    S = list(order[:npz])
    for t in range(npz, bh):
        red = np.maximum(0.0, cos[:, S].max(axis=1)) if S else np.zeros(nh)
        gt = s64[:nh] - lam * red
        gt[S] = -np.inf
        i = int(order[t])
        scale = np.abs(s64[i]) + lam * red[i]
        assert gt.max() - gt[i] <= P.NEAR_TIE * max(scale, 1e-30), (hh, t)
        assert abs(gain[t] - gt[i]) <= P.GAIN_RTOL * max(scale, 1e-30), (hh, t)
        S.append(i)
    assert len(ref["order"]) == bh - npz
    np.testing.assert_array_equal(_bits(out.K_out[hh])[:bh], O.compact(_bits(K[hh]), idx[:bh]))
    np.testing.assert_array_equal(_bits(out.V_out[hh])[:bh], O.compact(_bits(V[hh]), idx[:bh]))
    if pos is not None:
        np.testing.assert_array_equal(out.pos_out[hh].cpu().numpy()[:bh], pos[hh].numpy()[idx[:bh]])
        assert np.all(out.pos_out[hh].cpu().numpy()[bh:] == -1)


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_seeded_sweep_of_the_budget_allocator_frame(seed):
    # random head lengths, budgets, candidate counts, protected sets, per-head lambdas, dtypes and head
    # counts (a few heads: the single-event kernels; hundreds: the batched ones)
    rng = np.random.default_rng(seed)
    for case in range(14):
        dtype = torch.bfloat16 if rng.random() < 0.8 else torch.float32
        n = int(rng.choice([rng.integers(8, 130), rng.integers(130, 257), rng.integers(257, 1500 if dtype == torch.bfloat16 else 400)]))
        b_max = int(rng.integers(1, min(n, 200) + 1))
        h = int(rng.choice([1, 3, 7, 280])) if n <= 256 else int(rng.choice([1, 3, 6]))
        lam = float(rng.choice([0.0, 0.1, 0.5, 1.0]))
        g = torch.Generator().manual_seed(int(rng.integers(1 << 30)))
        K = torch.randn((h, n, 128), generator=g).to(dtype)
        V = torch.randn((h, n, 128), generator=g).to(dtype)
        if n > 4:
            V[:, n // 2:] = V[:, : n - n // 2] + 0.05 * V[:, n // 2:]
        s = torch.randn((h, n), generator=g).exp()
        n_h = torch.from_numpy(rng.integers(1, n + 1, size=h).astype(np.int32))
        if rng.random() < 0.3:
            n_h[:] = n
        b_h = torch.from_numpy(np.minimum(rng.integers(0, b_max + 1, size=h), n_h.numpy()).astype(np.int32))
        keep = torch.zeros((h, n), dtype=torch.uint8)
        for hh in range(h):
            cnt = int(rng.integers(0, int(b_h[hh]) + 1)) if rng.random() < 0.6 else 0
            if cnt:
                keep[hh, torch.from_numpy(rng.choice(int(n_h[hh]), size=cnt, replace=False))] = 1
        use_lam_h = lam > 0 and rng.random() < 0.4
        lam_h = torch.from_numpy(rng.choice([0.1, 0.5, 2.0], size=h).astype(np.float32)) if use_lam_h else None
        pos = torch.from_numpy(rng.integers(0, 1 << 20, size=(h, n)).astype(np.int32)) if rng.random() < 0.5 else None
        out = B().kvr_retain_budgeted(K.to(DEV), V.to(DEV), b_max, lam, 1e-6, s=s.to(DEV), n_h=n_h.to(DEV),
                                      b_h=b_h.to(DEV), keep=keep.to(DEV), pos=None if pos is None else pos.to(DEV),
                                      lam_h=None if lam_h is None else lam_h.to(DEV))
        torch.cuda.synchronize()
        heads = range(h) if h <= 7 else sorted(rng.choice(h, size=6, replace=False).tolist())
        for hh in heads:
            lh = float(lam_h[hh]) if use_lam_h else lam
            try:
                _check_budgeted_head(out, hh, K, V, W.to_f64(s[hh]), int(n_h[hh]), int(b_h[hh]),
                                     keep[hh].numpy().astype(bool), lh, pos)
            except AssertionError as e:
                raise AssertionError(f"case {case}: n={n} b_max={b_max} heads={h} head {hh} n_h={int(n_h[hh])} "
                                     f"b_h={int(b_h[hh])} lambda={lh} {dtype}: {e}") from e
