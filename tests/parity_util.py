"""Comparison of the HIP path's picks with the fp64 oracle.

The bar:
  * index sets and pick order equal to the free-running oracle's, except at
    picks where the oracle's best two marginal gains are within NEAR_TIE
    (relative) of each other; after such a pick the two runs may legitimately
    continue on different prefixes, so every pick of the HIP path is checked
    against the oracle's Eq. 2 evaluated on the HIP path's own prefix (it must be
    the fp64 argmax, or within NEAR_TIE of it);
  * gains within GAIN_RTOL relative; scores within SCORE_RTOL relative;
  * compacted rows bit-exact.
"Relative" for a gain s_i - lambda*m_i is taken against the magnitude of its
operands, |s_i| + lambda*m_i, because fp32 evaluates the difference with an
absolute error of an ulp of the operands, not of the (possibly cancelling)
result.
"""
from __future__ import annotations

import dataclasses

import numpy as np

from oracle import alpha_oracle as O

NEAR_TIE = 1e-5
GAIN_RTOL = 1e-4
SCORE_RTOL = 1e-4


@dataclasses.dataclass
class HeadReport:
    identical_to_free_run: bool
    near_ties: int            # picks of the HIP path that were not the fp64 argmax but within NEAR_TIE
    oracle_near_ties: int     # picks of the free-running oracle whose top two gains are within NEAR_TIE
    max_gain_err: float       # max |gain_hip - gain_fp64| / operand magnitude


def check_head(s64, V64, b, lam, eps, order, gain, idx_sorted) -> HeadReport:
    """Raises AssertionError when the HIP path's picks for one head are not valid."""
    s64 = np.asarray(s64, dtype=np.float64)
    n = s64.shape[0]
    order = np.asarray(order).astype(np.int64)
    gain = np.asarray(gain).astype(np.float64)
    idx_sorted = np.asarray(idx_sorted).astype(np.int64)
    assert order.shape == (b,) and idx_sorted.shape == (b,)
    assert order.min() >= 0 and order.max() < n, "pick out of range"
    assert len(set(order.tolist())) == b, "picks are not unique"
    assert idx_sorted.tolist() == sorted(order.tolist()), "idx_sorted != sort(pick_order)"

    free = O.alpha_select(s64, V64, b, lam, eps)
    fscale = np.maximum(np.abs(free["gain"]), np.abs(free["second"]))
    fscale = np.where(np.isfinite(fscale), fscale, 1.0)
    with np.errstate(invalid="ignore"):
        o_ties = int(np.sum((free["gain"] - free["second"]) <= NEAR_TIE * np.maximum(fscale, 1e-30)))
    identical = order.tolist() == free["order"].tolist()

    near = 0
    max_err = 0.0
    if lam == 0.0:
        # top-b: pick t must carry the t-th largest score (ties to the lower index)
        for t in range(b):
            g = order[t]
            mask = np.ones(n, bool)
            mask[order[:t]] = False
            best = s64[mask].max()
            scale = max(abs(best), abs(s64[g]), 1e-30)
            if order[t] != free["order"][t]:
                assert best - s64[g] <= NEAR_TIE * scale, f"top-b pick {t} is not a maximum"
                near += 1
            max_err = max(max_err, abs(gain[t] - s64[g]) / scale)
        assert max_err <= GAIN_RTOL
        return HeadReport(identical, near, o_ties, max_err)

    Vh = O.signatures(V64, eps)
    m = np.zeros(n)
    taken = np.zeros(n, bool)
    for t in range(b):
        a = s64 - lam * m if t > 0 else s64.copy()
        scale_all = np.abs(s64) + (lam * m if t > 0 else 0.0)
        a[taken] = -np.inf
        i_best = int(np.flatnonzero(a == a.max())[0])
        g = int(order[t])
        scale = max(scale_all[g], scale_all[i_best], 1e-30)
        if g != i_best:
            assert a[i_best] - a[g] <= NEAR_TIE * scale, (
                f"pick {t}: token {g} gain {a[g]!r} but token {i_best} has {a[i_best]!r}")
            near += 1
        err = abs(gain[t] - a[g]) / scale
        assert err <= GAIN_RTOL, f"pick {t}: gain {gain[t]!r} vs fp64 {a[g]!r}"
        max_err = max(max_err, err)
        taken[g] = True
        np.maximum(m, Vh @ Vh[g], out=m)
    if not identical:
        assert near > 0 or o_ties > 0, "sets differ from the free-running oracle without a near-tie"
    return HeadReport(identical, near, o_ties, max_err)


def check_scores(s_hip, s64):
    s_hip = np.asarray(s_hip, dtype=np.float64)
    err = np.abs(s_hip - s64) / np.maximum(np.abs(s64), 1e-30)
    assert err.max() <= SCORE_RTOL, f"score rel err {err.max()}"
    return float(err.max())


def summarize(reports):
    return dict(heads=len(reports),
                identical=sum(r.identical_to_free_run for r in reports),
                near_ties=sum(r.near_ties for r in reports),
                oracle_near_ties=sum(r.oracle_near_ties for r in reports),
                max_gain_err=max(r.max_gain_err for r in reports))


# ---------------------------------------------------------------------------
# jobs for a process pool (the benchmark's oracle legs run heads in parallel on
# the host cores; every argument and result is plain numpy / python).  Cached
# rows travel in the device format (bf16 bit patterns as int16, or float32) and
# are widened exactly inside the worker, before anything is timed.
# ---------------------------------------------------------------------------
def _widen(x):
    x = np.asarray(x)
    if x.dtype == np.int16:
        return O.bf16_bits_to_f64(x.view(np.uint16))
    return x.astype(np.float64)


def oracle_event_job(job):
    """One head's whole event on the oracle (score unless given, selection,
    compaction of K and V); returns the seconds it took inside the worker."""
    import time
    K, V = _widen(job["K"]), _widen(job["V"])
    Q = _widen(job["Q"]) if job.get("Q") is not None else None
    s = _widen(job["s"]) if job.get("s") is not None else None
    mode = job.get("mode", "plain")
    t0 = time.perf_counter()
    if mode == "flat":
        O.retain_flat(K, V, s, job["b"], job["lam"], job["eps"])
    elif mode == "budgeted":
        s64 = s if Q is None else O.score_softmax_mean(K, Q)
        r = O.select_budgeted(s64, V, job["n_h"], job["b"], job["keep"], job["lam"], job["eps"])
        O.compact(K, r["sorted"]); O.compact(V, r["sorted"])
    else:
        r = O.retain(K, V, job["b"], job["lam"], job["eps"], Q=Q, s=s)
        O.compact(K, r["sorted"]); O.compact(V, r["sorted"])
    return time.perf_counter() - t0


def check_head_job(job):
    """check_head for one head of a finished HIP run, plus the score comparison and the bitwise
    comparison of the kept rows; returns the HeadReport as a dict (raises on a mismatch)."""
    K, V = _widen(job["K"]), _widen(job["V"])
    score_err = 0.0
    if job.get("Q") is not None:
        s64 = O.score_softmax_mean(K, _widen(job["Q"]))
        score_err = check_scores(job["s_hip"], s64)
    else:
        s64 = _widen(job["s"])
    rep = check_head(s64, V, job["b"], job["lam"], job["eps"], job["order"], job["gain"], job["idx"])
    for X, X_out in ((job["K"], job["K_out"]), (job["V"], job["V_out"])):       # bit patterns, not values
        X, X_out = np.asarray(X), np.asarray(X_out)
        if X.dtype == np.float32:
            X, X_out = X.view(np.int32), X_out.view(np.int32)
        np.testing.assert_array_equal(X_out, O.compact(X, job["idx"]))
    d = dataclasses.asdict(rep)
    d["score_err"] = score_err
    return d
