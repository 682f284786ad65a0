"""Plain fp64 oracle of the per-compression-event retention step.

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke entry and by the
CPU-baseline leg of the benchmark; never by the product path.  It shares no
code with the HIP library and does not import it.

What is computed, and where the paper defines it (Sec. 4.1 "Method: A V-Space
Diversity Penalty"):

* V-signatures: each value row scaled by 1/(||row||_2 + eps)        (Eq. 1,
  with one layer and one head per problem: every (sequence, layer, KV-head)
  is its own selection problem).
* cosine of two signatures = their dot product                      (text
  after Eq. 1).
* marginal gain  s_i - lambda * max(0, max_{j in S} cos(v_i, v_j))  (Eq. 2).
* greedy fill: first pick argmax s, then argmax of the marginal gain over
  the unselected tokens, k-1 times                                  (Eq. 3).
* Algorithm 1 is that rule with the inner maximum of Eq. 2 carried along as
  a running vector (zero for the empty set, which is the max(0, .) floor);
  lambda == 0 returns top-k(s) through an explicit branch; the result is the
  sorted index set.
* The cache after the event is the selected rows of K and V in ascending
  token order (Sec. 1: a budget-bounded subset of cached tokens is kept;
  Algorithm 1 returns sort(S)).

The paper's base scorer is external to it.  The stand-in used by the synthetic
workloads is the mean over G grouped queries of softmax_i(q_g . k_i / sqrt(d))
(`score_softmax_mean`), or scores handed in directly.

Readings taken where the paper is silent: ties in every argmax go to the
lowest token index (this makes the greedy loop at lambda = 0 coincide with a
stable top-k, as the text requires of the fast path); eps is added to the
norm; all n tokens are candidates.

Pins (tests/test_oracle_pins.py): worked cases derived by hand (one of them
with exactly tied gains), lambda = 0 against a stable sort, orthonormal /
identical / antipodal value rows (closed forms), exactly tied gains at
lambda > 0 against a sort by (score descending, index ascending) that does not
go through this module's argmax, an exhaustive from-scratch evaluation of
Eq. 2 on tiny inputs (`greedy_from_definition`, which keeps no running maximum
and no cosine matrix), the runner-up gain against a brute-force second best,
softmax rows summing to one and matching scipy, invariants (k unique indices,
first pick = argmax s, non-increasing pick gains).  No function here is
"parity unpinned".
"""
from __future__ import annotations

import numpy as np

NEG_INF = -np.inf


# --------------------------------------------------------------------------
# exact widening of the device formats
# --------------------------------------------------------------------------
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 bit patterns -> float64, exactly (bf16 is the top half
    of an IEEE binary32)."""
    b = np.ascontiguousarray(bits).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------
# base score stand-in
# --------------------------------------------------------------------------
def score_softmax_mean(K: np.ndarray, Q: np.ndarray) -> np.ndarray:
    """s_i = (1/G) sum_g softmax_i(q_g . k_i / sqrt(d)).  K [n,d], Q [G,d]."""
    K = np.asarray(K, dtype=np.float64)
    Q = np.asarray(Q, dtype=np.float64)
    n, d = K.shape
    z = (Q @ K.T) / np.sqrt(float(d))              # [G, n]
    z = z - z.max(axis=1, keepdims=True)
    p = np.exp(z)
    p = p / p.sum(axis=1, keepdims=True)
    return p.mean(axis=0)


# --------------------------------------------------------------------------
# Eq. 1
# --------------------------------------------------------------------------
def score_pool(s, kernel: int, mean: bool = False) -> np.ndarray:
    """Pooling of a score row over the window of `kernel` (odd) tokens centred on each token,
    the smoothing step of observation-window scorers (the scorer family of Sec. 2; the paper
    does not restate it).  Reading: positions outside the row are skipped by the maximum and
    count as zeros in the mean, whose divisor is always `kernel`."""
    s = np.asarray(s, dtype=np.float64)
    n, half = len(s), kernel // 2
    out = np.empty(n)
    for i in range(n):
        win = s[max(i - half, 0): min(i + half, n - 1) + 1]
        out[i] = win.sum() / kernel if mean else win.max()
    return out


def score_mean_direction_prior(s, V, lam_p: float, eps: float = 1e-6) -> np.ndarray:
    """The modular one-term variant the paper tested and rejected (table of negative gates,
    scoring family): s_i + lam_p * cos(V_i, dir), dir the mean of the head's value rows.
    Reading: the mean is over the head's n candidate rows, and both norms carry Eq. 1's eps."""
    V = np.asarray(V, dtype=np.float64)
    d = V.mean(axis=0)
    cos = (V @ d) / ((np.sqrt((V * V).sum(axis=1)) + eps) * (np.sqrt((d * d).sum()) + eps))
    return np.asarray(s, dtype=np.float64) + lam_p * cos


def signatures(V: np.ndarray, eps: float) -> np.ndarray:
    """v_i = u_i / (||u_i||_2 + eps), one layer and one head (u_i = V_i)."""
    V = np.asarray(V, dtype=np.float64)
    norm = np.sqrt((V * V).sum(axis=1, keepdims=True))
    return V / (norm + eps)


def signatures_flat(V_all: np.ndarray, eps: float) -> np.ndarray:
    """Eq. 1 as printed: u_i is the mean of V over all layers and heads.
    V_all [L*H, n, d]."""
    u = np.asarray(V_all, dtype=np.float64).mean(axis=0)
    return signatures(u, eps)


# --------------------------------------------------------------------------
# top-k (lambda = 0 branch of Algorithm 1)
# --------------------------------------------------------------------------
def _argmax_lowest(a: np.ndarray) -> int:
    """argmax with ties to the lowest index (numpy's argmax already returns
    the first maximum; spelled out because the reading matters)."""
    return int(np.flatnonzero(a == a.max())[0])


def topk_order(s: np.ndarray, k: int) -> np.ndarray:
    """The k largest scores in pick order (descending score, ties to the
    lower index)."""
    s = np.asarray(s, dtype=np.float64)
    order = np.argsort(-s, kind="stable")
    return order[:k].astype(np.int64)


# --------------------------------------------------------------------------
# the selector (Eq. 2 and Eq. 3; the rule Algorithm 1 implements)
# --------------------------------------------------------------------------
def alpha_select(s, V, k: int, lam: float, eps: float = 1e-6):
    """The greedy fill of Eq. 3 under the marginal gain of Eq. 2, in fp64.

    For the current set S every unselected token i is worth
    s_i - lam * max(0, max_{j in S} <v_i, v_j>)  (Eq. 2); the best one joins S
    (Eq. 3), k times, starting from the empty set, for which the inner term is
    the floor 0 and the first member is therefore argmax s.  The inner maximum
    is carried from one step to the next: when i joins S it gains exactly one
    term, <v_., v_i>, which is the one row of cosines computed per member (the
    n x n matrix of Algorithm 1 holds the same numbers; only k of its rows are
    ever looked at).  lam == 0 takes the explicit branch the paper requires of
    the selector: top-k of s, no value row is touched.

    Returns a dict with
      order   [k]  members in the order they joined,
      gain    [k]  Eq. 2 of each member when it joined (gain[0] is max s),
      second  [k]  the largest Eq. 2 value among the other unselected tokens
                   at that step (-inf when none is left),
      sorted  [k]  sort(S), the selector's return value.
    """
    s = np.asarray(s, dtype=np.float64)
    n = s.shape[0]
    if not (1 <= k <= n):
        raise ValueError("need 1 <= k <= n")
    if not (lam >= 0.0):
        raise ValueError("need lambda >= 0")
    order = np.empty(k, dtype=np.int64)
    gain = np.empty(k)
    second = np.full(k, NEG_INF)
    if lam == 0.0:
        order[:] = topk_order(s, k)
        gain[:] = s[order]
        by_value = np.sort(s)[::-1]
        second[: min(k, n - 1)] = by_value[1: min(k, n - 1) + 1]
        return dict(order=order, gain=gain, second=second, sorted=np.sort(order))
    Vh = signatures(V, eps)
    redundancy = np.zeros(n)            # Eq. 2's max(0, max_{j in S} <v_i, v_j>) for the current S
    free = np.ones(n, dtype=bool)
    for t in range(k):
        value = np.where(free, s - lam * redundancy, NEG_INF)      # Eq. 2
        i = _argmax_lowest(value)                                  # Eq. 3
        order[t], gain[t] = i, value[i]
        if n > 1:
            second[t] = np.delete(value, i).max()
        free[i] = False
        np.maximum(redundancy, Vh @ Vh[i], out=redundancy)         # S now holds i
    return dict(order=order, gain=gain, second=second, sorted=np.sort(order))


# --------------------------------------------------------------------------
# Eq. 2 / Eq. 3 written out with no running state (for tiny n)
# --------------------------------------------------------------------------
def marginal_gains(s, Vh, S, lam: float) -> np.ndarray:
    """Eq. 2 for every token given the selected list S (signatures Vh already
    unit-normalised); selected tokens get -inf.  Nothing incremental: the
    inner maximum is recomputed over the whole of S."""
    s = np.asarray(s, dtype=np.float64)
    n = s.shape[0]
    out = np.empty(n)
    Sset = set(int(j) for j in S)
    for i in range(n):
        if i in Sset:
            out[i] = NEG_INF
            continue
        red = 0.0
        if len(S):
            red = max(0.0, max(float(np.dot(Vh[i], Vh[j])) for j in S))
        out[i] = s[i] - lam * red
    return out


def greedy_from_definition(s, V, k: int, lam: float, eps: float = 1e-6):
    """Eq. 3 with Eq. 2 evaluated from scratch at every step."""
    s = np.asarray(s, dtype=np.float64)
    Vh = signatures(V, eps)
    S = [_argmax_lowest(s)]
    gains = [float(s[S[0]])]
    for _ in range(1, k):
        g = marginal_gains(s, Vh, S, lam)
        i = _argmax_lowest(g)
        S.append(i)
        gains.append(float(g[i]))
    return np.asarray(S, dtype=np.int64), np.asarray(gains)


# --------------------------------------------------------------------------
# cache update
# --------------------------------------------------------------------------
def compact(X: np.ndarray, idx_sorted: np.ndarray) -> np.ndarray:
    """Rows of X at the ascending indices, bit for bit (X may be a raw
    integer view of the device format)."""
    return np.ascontiguousarray(np.asarray(X)[np.asarray(idx_sorted)])


def compact_inplace(X: np.ndarray, idx_sorted: np.ndarray) -> np.ndarray:
    """The cache update done in the cache's own rows, one row after the other as a serving
    loop would: row t receives row idx_sorted[t], lowest t first; entries < 0 move nothing and
    rows past the list keep their contents.  For the strictly ascending list Algorithm 1
    returns (sort(S), so idx_sorted[t] >= t) no source row has been overwritten when it is
    read, and the front of the result equals compact(X, idx_sorted)."""
    Y = np.array(X, copy=True)
    for t, i in enumerate(np.asarray(idx_sorted).tolist()):
        if i >= 0:
            Y[t] = Y[i]
    return Y


def retain(K, V, k: int, lam: float, eps: float = 1e-6, Q=None, s=None):
    """Whole event for one head: score (unless given), select, and the
    sorted index set.  K, V are float64 views of the cached rows."""
    if s is None:
        s = score_softmax_mean(K, Q)
    sel = alpha_select(s, V, k, lam, eps)
    sel["s"] = np.asarray(s, dtype=np.float64)
    return sel


def retain_flat(K_all, V_all, s, k: int, lam: float, eps: float = 1e-6):
    """Flat-signature event (Eq. 1 as printed, then Algorithm 1 once per sequence): the
    signature rows are the mean of V over all L*H heads, one selection from one score vector,
    and every head keeps the same token set.  K_all, V_all [L*H, n, d]; s [n]."""
    V_all = np.asarray(V_all, dtype=np.float64)
    u = V_all.mean(axis=0)                       # Eq. 1 before the normalisation
    r = alpha_select(s, u, k, lam, eps)          # normalises u inside (Eq. 1), then Eq. 2-3
    r["u"] = u
    r["K_out"] = np.stack([compact(Kh, r["sorted"]) for Kh in np.asarray(K_all)])
    r["V_out"] = np.stack([compact(Vh, r["sorted"]) for Vh in np.asarray(V_all)])
    return r


def select_budgeted(s, V, n_h: int, b_h: int, keep=None, lam: float = 0.5, eps: float = 1e-6):
    """Algorithm 1 inside a budget allocator's frame: only the first n_h tokens are candidates,
    the tokens flagged in `keep` (sinks, recent window) are members of S from the start and count
    towards the budget b_h, and the greedy fill of Eq. 3 continues from there until |S| = b_h.
    Eq. 2 is evaluated from scratch at every step (no running state).  Returns the protected
    tokens (ascending), the greedy picks in pick order with their gains, and sort(S)."""
    s = np.asarray(s, dtype=np.float64)[:n_h]
    Vh = signatures(np.asarray(V, dtype=np.float64)[:n_h], eps)
    prot = [] if keep is None else [int(j) for j in np.flatnonzero(np.asarray(keep)[:n_h])]
    if len(prot) > b_h:
        raise ValueError("more protected tokens than budget")
    S = list(prot)
    order, gain = [], []
    cos = Vh @ Vh.T
    while len(S) < b_h:
        red = np.maximum(0.0, cos[:, S].max(axis=1)) if S else np.zeros(len(s))   # Eq. 2's inner maximum over all of S
        g = s - lam * red
        g[S] = NEG_INF
        i = _argmax_lowest(g)
        order.append(i); gain.append(g[i]); S.append(i)
    return {"protected": np.array(prot, dtype=np.int64), "order": np.array(order, dtype=np.int64),
            "gain": np.array(gain, dtype=np.float64), "sorted": np.array(sorted(S), dtype=np.int64)}

