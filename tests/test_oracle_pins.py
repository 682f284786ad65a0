"""Pins of the fp64 oracle against what the paper and the mathematics fix
(Sec. 4.1: Eq. 1-3, Algorithm 1).  CPU only."""
import itertools
import json
import os

import numpy as np
import pytest
import scipy.special

from oracle import alpha_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- hand cases
def test_hand_case_five_tokens():
    g = json.load(open(os.path.join(GOLD, "hand_case.json")))
    r = O.alpha_select(g["s"], np.array(g["V"]), g["k"], g["lambda"], g["eps"])
    assert r["order"].tolist() == g["order"]
    np.testing.assert_allclose(r["gain"], g["gain"], rtol=0, atol=1e-12)
    assert r["sorted"].tolist() == g["sorted"]


def test_hand_case_four_tokens_two_lambdas():
    g = json.load(open(os.path.join(GOLD, "hand_case.json")))["second_case"]
    for c in g["cases"]:
        r = O.alpha_select(g["s"], np.array(g["V"]), g["k"], c["lambda"], g["eps"])
        assert r["order"].tolist() == c["order"]
        np.testing.assert_allclose(r["gain"], c["gain"], atol=1e-12)


def test_hand_case_with_exactly_tied_gains():
    g = json.load(open(os.path.join(GOLD, "hand_case.json")))["tied_case"]
    r = O.alpha_select(g["s"], np.array(g["V"]), g["k"], g["lambda"], g["eps"])
    assert r["order"].tolist() == g["order"]
    assert r["gain"].tolist() == g["gain"]
    assert r["second"].tolist() == g["second"]
    assert r["sorted"].tolist() == g["sorted"]
    order, gains = O.greedy_from_definition(g["s"], np.array(g["V"]), g["k"], g["lambda"], g["eps"])
    assert order.tolist() == g["order"] and gains.tolist() == g["gain"]


# ------------------------------------------ the tie rule: lowest token index
# Expected values below never go through the oracle's own argmax helper: they are
# sorted(range(n), key=(-score, index)), written out.
def _by_score_then_index(s, k):
    return sorted(range(len(s)), key=lambda i: (-s[i], i))[:k]


@pytest.mark.parametrize("lam", [0.25, 1.0])
@pytest.mark.parametrize("seed", range(4))
def test_tied_scores_on_orthonormal_rows_join_in_index_order(seed, lam):
    # orthonormal rows: every cosine is exactly 0, so Eq. 2 is the score and the
    # greedy loop must walk the tokens by (score descending, index ascending)
    rng = _rng(300 + seed)
    n, k = 24, 17
    s = rng.integers(0, 4, n).astype(np.float64)        # four levels: many exact ties
    V = np.eye(n)
    expect = _by_score_then_index(s, k)
    r = O.alpha_select(s, V, k, lam, 0.0)
    assert r["order"].tolist() == expect
    assert r["gain"].tolist() == [s[i] for i in expect]
    order, _ = O.greedy_from_definition(s, V, k, lam, 0.0)
    assert order.tolist() == expect
    b = O.select_budgeted(s, V, n, k, None, lam, 0.0)
    assert b["order"].tolist() == expect


@pytest.mark.parametrize("lam", [0.25, 1.0])
def test_tied_scores_on_identical_rows_join_in_index_order(lam):
    # identical unit rows, eps = 0: after the first member every value is score - lam exactly
    # (quarter-integer scores and these lambdas are exact in binary), so the order is again
    # (score descending, index ascending), with ties at every level
    rng = _rng(17)
    n, k = 30, 21
    s = rng.integers(0, 5, n) / 4.0
    V = np.tile(np.array([[0.0, 1.0, 0.0]]), (n, 1))
    expect = _by_score_then_index(s, k)
    r = O.alpha_select(s, V, k, lam, 0.0)
    assert r["order"].tolist() == expect
    assert r["gain"].tolist() == [s[expect[0]]] + [s[i] - lam for i in expect[1:]]
    order, _ = O.greedy_from_definition(s, V, k, lam, 0.0)
    assert order.tolist() == expect


def test_first_member_tie_goes_to_the_lowest_index():
    s = np.array([1.0, 3.0, 3.0, 2.0, 3.0])
    V = _rng(2).normal(size=(5, 3))
    assert O.alpha_select(s, V, 1, 0.5)["order"].tolist() == [1]
    assert O.alpha_select(s, V, 1, 0.0)["order"].tolist() == [1]
    assert O.greedy_from_definition(s, V, 1, 0.5)[0].tolist() == [1]
    assert O.select_budgeted(s, V, 5, 1)["order"].tolist() == [1]


def test_greedy_loop_at_lambda_zero_is_the_stable_topk():
    # the loop form of Eq. 3 with lam = 0 (no fast path) on heavily tied scores
    rng = _rng(23)
    n, k = 60, 33
    s = rng.integers(0, 6, n).astype(np.float64)
    V = rng.normal(size=(n, 5))
    expect = _by_score_then_index(s, k)
    assert O.greedy_from_definition(s, V, k, 0.0)[0].tolist() == expect
    assert O.topk_order(s, k).tolist() == expect
    assert O.select_budgeted(s, V, n, k, None, 0.0)["order"].tolist() == expect


def test_budgeted_frame_breaks_ties_among_free_tokens_towards_the_lowest_index():
    # token 0 protected (row e1); free tokens 1..4: rows e2,e2,e3,e3, equal scores.
    # t0: values of 1..4 all 1.0 -> 1 joins; then 2 is penalised (1 - .5), 3 and 4 tie at 1.0 -> 3;
    # then 2 and 4 tie at .5 -> 2.
    E = np.eye(3)
    V = np.stack([E[0], E[1], E[1], E[2], E[2]])
    s = np.array([0.0, 1.0, 1.0, 1.0, 1.0])
    keep = np.array([1, 0, 0, 0, 0], dtype=np.uint8)
    r = O.select_budgeted(s, V, 5, 4, keep, 0.5, 0.0)
    assert r["protected"].tolist() == [0]
    assert r["order"].tolist() == [1, 3, 2]
    assert r["gain"].tolist() == [1.0, 1.0, 0.5]


@pytest.mark.parametrize("seed", range(6))
def test_runner_up_gain_is_the_brute_force_second_best(seed):
    rng = _rng(500 + seed)
    n = int(rng.integers(3, 11))
    V = rng.normal(size=(n, 4))
    s = rng.integers(0, 3, n) / 2.0 if seed % 2 else rng.uniform(0, 1, n)    # with and without ties
    lam, eps, k = 0.5, 1e-6, n
    r = O.alpha_select(s, V, k, lam, eps)
    Vh = O.signatures(V, eps)
    for t in range(k):
        S = r["order"][:t].tolist()
        vals = []
        for i in range(n):
            if i in S:
                continue
            red = max([0.0] + [float(Vh[i] @ Vh[j]) for j in S])
            vals.append(s[i] - lam * red)
        vals.sort(reverse=True)
        assert abs(vals[0] - r["gain"][t]) < 1e-13
        if len(vals) > 1:
            assert abs(vals[1] - r["second"][t]) < 1e-13 and r["second"][t] <= r["gain"][t]
        else:
            assert r["second"][t] == -np.inf
    z = O.alpha_select(s, V, k, 0.0)                 # the lambda = 0 branch reports the next score down
    by_value = sorted(s.tolist(), reverse=True)
    assert z["second"][: n - 1].tolist() == by_value[1:] and z["second"][n - 1] == -np.inf


def test_tie_pins_fail_when_ties_go_to_the_highest_index(monkeypatch):
    # the planted mistake: argmax returning the last maximum instead of the first
    monkeypatch.setattr(O, "_argmax_lowest", lambda a: int(np.flatnonzero(a == a.max())[-1]))
    for pin in (test_hand_case_with_exactly_tied_gains,
                lambda: test_tied_scores_on_orthonormal_rows_join_in_index_order(0, 0.25),
                lambda: test_tied_scores_on_identical_rows_join_in_index_order(1.0),
                test_first_member_tie_goes_to_the_lowest_index,
                test_greedy_loop_at_lambda_zero_is_the_stable_topk,
                test_budgeted_frame_breaks_ties_among_free_tokens_towards_the_lowest_index):
        with pytest.raises(AssertionError):
            pin()


# ------------------------------------------------- lambda = 0 is stable top-k
@pytest.mark.parametrize("seed", range(5))
def test_lambda_zero_is_stable_topk(seed):
    rng = _rng(seed)
    n, d, k = 97, 16, 31
    s = rng.integers(0, 12, n).astype(np.float64)      # many exact ties
    V = rng.normal(size=(n, d))
    r = O.alpha_select(s, V, k, 0.0)
    # independent statement of "k largest, ties to the lower index"
    expect = sorted(range(n), key=lambda i: (-s[i], i))[:k]
    assert r["order"].tolist() == expect
    assert r["sorted"].tolist() == sorted(expect)


def test_greedy_loop_at_tiny_lambda_matches_topk_when_gaps_are_large():
    # with score gaps of 1 and lambda = 1e-9 the loop (not the fast path) must
    # still give top-k: pins the loop's masking and the first pick
    rng = _rng(3)
    n, k = 40, 17
    s = rng.permutation(n).astype(np.float64)
    V = rng.normal(size=(n, 8))
    r = O.alpha_select(s, V, k, 1e-9)
    assert r["order"].tolist() == list(np.argsort(-s)[:k])


# ------------------------------------------------------------- closed forms
def test_orthonormal_rows_give_topk_for_any_lambda():
    rng = _rng(1)
    n = 24
    Qm, _ = np.linalg.qr(rng.normal(size=(32, 32)))
    V = Qm[:n] * rng.uniform(0.5, 3.0, size=(n, 1))     # orthogonal, any norm
    s = rng.normal(size=n)
    for lam in (0.25, 1.0, 5.0):
        r = O.alpha_select(s, V, 9, lam, eps=0.0)
        assert r["order"].tolist() == list(np.argsort(-s, kind="stable")[:9])
        np.testing.assert_allclose(r["gain"], np.sort(s)[::-1][:9], atol=1e-12)


def test_identical_rows_shift_every_later_gain_by_lambda():
    rng = _rng(2)
    n, k, lam = 30, 12, 0.7
    V = np.tile(rng.normal(size=(1, 8)), (n, 1))
    s = rng.normal(size=n)
    r = O.alpha_select(s, V, k, lam, eps=0.0)
    top = np.argsort(-s, kind="stable")[:k]
    assert r["order"].tolist() == top.tolist()
    np.testing.assert_allclose(r["gain"][0], s[top[0]], atol=1e-12)
    np.testing.assert_allclose(r["gain"][1:], s[top[1:]] - lam, atol=1e-12)


def test_antipodal_pairs_get_no_bonus():
    # rows x and -x: cosine -1 is floored to zero, so with mutually orthogonal
    # pairs the result is top-k
    n = 16
    V = np.zeros((n, 8))
    for p in range(8):
        V[2 * p, p] = 1.0
        V[2 * p + 1, p] = -1.0
    s = _rng(4).normal(size=n)
    r = O.alpha_select(s, V, 7, 0.9, eps=0.0)
    assert r["order"].tolist() == list(np.argsort(-s, kind="stable")[:7])


def test_k_equals_one_and_k_equals_n():
    rng = _rng(5)
    s = rng.normal(size=13)
    V = rng.normal(size=(13, 4))
    assert O.alpha_select(s, V, 1, 0.5)["order"].tolist() == [int(np.argmax(s))]
    assert O.alpha_select(s, V, 13, 0.5)["sorted"].tolist() == list(range(13))


# ------------------------------------------------ Eq. 2 from scratch, tiny n
@pytest.mark.parametrize("seed", range(12))
def test_algorithm1_equals_definition_on_tiny_inputs(seed):
    rng = _rng(100 + seed)
    n = int(rng.integers(2, 13))
    d = int(rng.integers(2, 6))
    V = rng.normal(size=(n, d))
    if seed % 3 == 0:                        # near-duplicate rows
        V[n // 2:] = V[: n - n // 2] + 0.05 * rng.normal(size=(n - n // 2, d))
    s = rng.normal(size=n) if seed % 2 else rng.uniform(0, 0.02, size=n)
    for lam in (0.25, 0.5, 1.0, 1.5):
        for k in range(1, n + 1):
            a = O.alpha_select(s, V, k, lam)
            order, gains = O.greedy_from_definition(s, V, k, lam)
            assert a["order"].tolist() == order.tolist()
            np.testing.assert_allclose(a["gain"], gains, atol=1e-13)


def test_each_pick_is_the_exhaustive_argmax():
    # for every prefix of the pick list, every unselected token's Eq. 2 value
    # is <= the gain of the token that was picked (and ties go low)
    rng = _rng(42)
    n, k, lam, eps = 11, 8, 0.5, 1e-6
    V = rng.normal(size=(n, 3))
    s = rng.uniform(0, 0.5, size=n)
    r = O.alpha_select(s, V, k, lam, eps)
    Vh = O.signatures(V, eps)
    for t in range(1, k):
        S = r["order"][:t].tolist()
        best, arg = -np.inf, None
        for i in range(n):
            if i in S:
                continue
            red = max([0.0] + [float(Vh[i] @ Vh[j]) for j in S])
            g = s[i] - lam * red
            if g > best:
                best, arg = g, i
        assert arg == r["order"][t]
        assert abs(best - r["gain"][t]) < 1e-13


# ----------------------------------------------------------------- invariants
@pytest.mark.parametrize("seed", range(4))
def test_invariants(seed):
    rng = _rng(200 + seed)
    n, d, k = 150, 32, 60
    V = rng.normal(size=(n, d))
    V[50:100] = V[:50] + 0.05 * rng.normal(size=(50, d))
    s = rng.lognormal(size=n)
    r = O.alpha_select(s, V, k, 0.5)
    assert len(set(r["order"].tolist())) == k
    assert r["order"].min() >= 0 and r["order"].max() < n
    assert r["order"][0] == int(np.argmax(s))
    assert np.all(np.diff(r["gain"]) <= 1e-15)            # non-increasing
    assert np.all(r["second"] <= r["gain"] + 1e-15)
    assert r["sorted"].tolist() == sorted(r["order"].tolist())


def test_positive_row_scaling_leaves_picks_unchanged():
    rng = _rng(7)
    n, d, k = 80, 16, 30
    V = rng.normal(size=(n, d))
    s = rng.uniform(0, 0.02, size=n)
    a = O.alpha_select(s, V, k, 0.5, eps=0.0)
    scale = 2.0 ** rng.integers(-6, 7, size=(n, 1))
    b = O.alpha_select(s, V * scale, k, 0.5, eps=0.0)
    assert a["order"].tolist() == b["order"].tolist()


def test_signatures_norm_and_eps_reading():
    rng = _rng(8)
    V = rng.normal(size=(9, 5))
    V[3] = 0.0
    eps = 1e-3
    Vh = O.signatures(V, eps)
    nv = np.linalg.norm(V, axis=1)
    np.testing.assert_allclose(np.linalg.norm(Vh, axis=1), nv / (nv + eps), atol=1e-14)
    assert np.all(Vh[3] == 0.0)             # zero row stays zero, never penalised
    flat = O.signatures_flat(np.stack([V[:3], 3 * V[:3]]), 0.0)
    np.testing.assert_allclose(flat, O.signatures(V[:3], 0.0), atol=1e-14)


def test_cosine_matrix_properties():
    rng = _rng(9)
    Vh = O.signatures(rng.standard_t(3, size=(40, 16)), 0.0)
    S = Vh @ Vh.T
    np.testing.assert_allclose(S, S.T, atol=1e-15)
    np.testing.assert_allclose(np.diag(S), 1.0, atol=1e-14)
    assert np.abs(S).max() <= 1 + 1e-14


# ----------------------------------------------------------------- base score
def test_score_is_mean_of_softmax_rows():
    rng = _rng(10)
    n, d, G = 50, 16, 7
    K = rng.normal(size=(n, d))
    Q = rng.normal(size=(G, d))
    s = O.score_softmax_mean(K, Q)
    assert abs(s.sum() - 1.0) < 1e-14
    ref = scipy.special.softmax(Q @ K.T / 4.0, axis=1).mean(axis=0)
    np.testing.assert_allclose(s, ref, rtol=1e-13)
    # one query: plain softmax; by hand for a two-token case
    s2 = O.score_softmax_mean(np.array([[2.0, 0.0], [0.0, 0.0]]), np.array([[np.sqrt(2.0), 0.0]]))
    np.testing.assert_allclose(s2, [np.e**2 / (np.e**2 + 1), 1 / (np.e**2 + 1)], rtol=1e-14)
    # logits far beyond exp's range must not overflow (max-subtraction)
    big = O.score_softmax_mean(np.array([[4000.0, 0.0], [0.0, 0.0]]), np.array([[4000.0, 0.0]]))
    np.testing.assert_allclose(big, [1.0, 0.0], atol=1e-300)


# ------------------------------------------------------------ format / compact
def test_bf16_widening_is_exact():
    bits = np.array([0x3F80, 0xBF80, 0x0000, 0x4049, 0x7F7F, 0x0080], dtype=np.uint16)
    want = [1.0, -1.0, 0.0, 3.140625, 3.3895313892515355e38, 2.0 ** -126]
    np.testing.assert_array_equal(O.bf16_bits_to_f64(bits), want)


def test_compact_is_a_row_gather():
    X = np.arange(40, dtype=np.uint16).reshape(10, 4)
    idx = np.array([1, 4, 9])
    out = O.compact(X, idx)
    assert out.tolist() == [X[1].tolist(), X[4].tolist(), X[9].tolist()]
    assert O.compact(out, np.arange(3)).tolist() == out.tolist()


# ---------------------------------------- a planted mistake must break a pin

def test_inplace_compaction_equals_the_gather_for_ascending_lists():
    rng = np.random.default_rng(5)
    for n, b in [(1, 1), (7, 7), (40, 13), (64, 1), (200, 199)]:
        X = rng.integers(0, 1 << 16, size=(n, 4))
        idx = np.sort(rng.choice(n, size=b, replace=False))
        Y = O.compact_inplace(X, idx)
        assert Y[:b].tolist() == X[idx].tolist()          # the textbook gather
        assert Y[b:].tolist() == X[b:].tolist()           # the tail is not touched
    # padding moves nothing; a shift by one is the case where every destination is the previous source
    X = np.arange(12).reshape(6, 2)
    assert O.compact_inplace(X, np.array([1, 4, -1, -1]))[:, 0].tolist() == [2, 8, 4, 6, 8, 10]
    assert O.compact_inplace(X, np.arange(1, 6))[:, 0].tolist() == [2, 4, 6, 8, 10, 10]
    # the precondition matters: a descending list reads rows that were already replaced
    assert O.compact_inplace(X, np.array([1, 0]))[:2, 0].tolist() != X[[1, 0], 0].tolist()

def test_pins_catch_planted_mistakes(monkeypatch):
    g = json.load(open(os.path.join(GOLD, "hand_case.json")))
    V = np.array(g["V"])

    def no_floor(s, V, k, lam, eps=1e-6):
        s = np.asarray(s, float)
        Vh = O.signatures(V, eps)
        sims = Vh @ Vh.T
        m = np.full(len(s), -np.inf)             # mistake: m not floored at 0
        sel, order = np.zeros(len(s), bool), []
        a = s.copy()
        for _ in range(k):
            i = int(np.argmax(a)); order.append(i); sel[i] = True
            m = np.maximum(m, sims[i])
            a = s - lam * m; a[sel] = -np.inf
        return order

    assert no_floor(g["s"], V, g["k"], g["lambda"], 0.0) != g["order"]


# ---------------------------------------------------------------- flat-signature mode (Eq. 1 over L*H)
def test_flat_mode_with_one_head_is_the_per_head_selection():
    rng = _rng(21)
    V = rng.normal(size=(1, 30, 8)); K = rng.normal(size=(1, 30, 8)); s = rng.random(30)
    f = O.retain_flat(K, V, s, 9, 0.6)
    r = O.alpha_select(s, V[0], 9, 0.6)
    assert f["order"].tolist() == r["order"].tolist()
    np.testing.assert_array_equal(f["K_out"][0], K[0][r["sorted"]])


def test_flat_mode_reproduces_the_hand_case_from_two_heads():
    # two heads whose mean is the hand case's V: V +/- D averages to V exactly
    g = json.load(open(os.path.join(GOLD, "hand_case.json")))
    V = np.array(g["V"])
    D = _rng(3).integers(-4, 5, size=V.shape).astype(np.float64)
    f = O.retain_flat(np.zeros((2,) + V.shape), np.stack([V + D, V - D]), g["s"], g["k"], g["lambda"], g["eps"])
    assert f["order"].tolist() == g["order"]
    np.testing.assert_allclose(f["gain"], g["gain"], rtol=0, atol=1e-12)


def test_flat_mode_cancelling_heads_give_plain_topk():
    # V and -V average to zero rows: zero signatures, no penalty, Eq. 3 is top-k of s
    rng = _rng(22)
    V = rng.normal(size=(20, 6)); s = rng.random(20)
    f = O.retain_flat(np.zeros((2, 20, 6)), np.stack([V, -V]), s, 7, 0.9)
    assert f["order"].tolist() == O.topk_order(s, 7).tolist()
    np.testing.assert_allclose(f["gain"], np.sort(s)[::-1][:7], rtol=0, atol=0)


def test_flat_mode_ignores_head_order_and_common_scale_and_shares_the_index_set():
    rng = _rng(23)
    V = rng.normal(size=(4, 25, 8)); K = rng.normal(size=(4, 25, 8)); s = rng.random(25)
    f = O.retain_flat(K, V, s, 10, 0.5)
    p = [2, 0, 3, 1]
    assert O.retain_flat(K[p], V[p], s, 10, 0.5)["order"].tolist() == f["order"].tolist()
    assert O.retain_flat(K, 8.0 * V, s, 10, 0.5, eps=0.0)["order"].tolist() == \
        O.retain_flat(K, V, s, 10, 0.5, eps=0.0)["order"].tolist()
    for h in range(4):
        np.testing.assert_array_equal(f["K_out"][h], K[h][f["sorted"]])
        np.testing.assert_array_equal(f["V_out"][h], V[h][f["sorted"]])
    # the mean, not the sum of per-head signatures: a head with huge rows dominates u
    big = V.copy(); big[0] *= 1e6
    assert O.retain_flat(K, big, s, 10, 0.5)["order"].tolist() == O.alpha_select(s, big[0], 10, 0.5)["order"].tolist()


# ---------------------------------------------------------------- budgets and protected tokens
def test_budgeted_without_protection_is_algorithm1_and_a_prefix_for_smaller_budgets():
    rng = _rng(31)
    V = rng.normal(size=(40, 8)); s = rng.random(40)
    full = O.alpha_select(s, V, 15, 0.6)
    r = O.select_budgeted(s, V, 40, 15, None, 0.6)
    assert r["order"].tolist() == full["order"].tolist()
    np.testing.assert_allclose(r["gain"], full["gain"], rtol=0, atol=1e-12)
    assert O.select_budgeted(s, V, 40, 6, None, 0.6)["order"].tolist() == full["order"][:6].tolist()
    # only the first n_h tokens are candidates: the same as running on the truncated arrays
    t = O.select_budgeted(s, V, 25, 10, None, 0.6)
    assert t["order"].tolist() == O.alpha_select(s[:25], V[:25], 10, 0.6)["order"].tolist()


def test_budgeted_gains_follow_eq2_with_the_protected_set_included():
    rng = _rng(32)
    V = rng.normal(size=(30, 6)); s = rng.random(30)
    keep = np.zeros(30, dtype=bool); keep[[0, 1, 28, 29]] = True        # sinks and a recent window
    r = O.select_budgeted(s, V, 30, 12, keep, 0.8)
    assert r["protected"].tolist() == [0, 1, 28, 29] and len(r["order"]) == 8
    assert set(r["protected"]) <= set(r["sorted"]) and len(set(r["sorted"].tolist())) == 12
    Vh = O.signatures(V, 1e-6)
    S = list(r["protected"])
    for i, g in zip(r["order"], r["gain"]):
        ref = O.marginal_gains(s, Vh, S, 0.8)        # the plain-loop form of Eq. 2
        assert i == int(np.flatnonzero(ref == ref.max())[0]) and abs(ref[i] - g) < 1e-12
        S.append(int(i))


def test_protecting_what_greedy_picks_first_changes_nothing_and_duplicates_of_protected_rows_are_penalised():
    rng = _rng(33)
    V = rng.normal(size=(30, 6)); s = rng.random(30)
    full = O.alpha_select(s, V, 10, 0.5)
    keep = np.zeros(30, dtype=bool); keep[full["order"][:4]] = True
    r = O.select_budgeted(s, V, 30, 10, keep, 0.5)
    assert r["order"].tolist() == full["order"][4:].tolist()
    assert r["sorted"].tolist() == full["sorted"].tolist()
    # a copy of a protected row carries the full penalty from the first greedy step on
    V2 = V.copy(); V2[7] = V2[0]; s2 = s.copy(); s2[7] = s.max() + 0.1
    keep2 = np.zeros(30, dtype=bool); keep2[0] = True
    r2 = O.select_budgeted(s2, V2, 30, 3, keep2, 2.0)
    assert 7 not in r2["order"].tolist()
    assert O.select_budgeted(s2, V2, 30, 3, keep2, 0.0)["order"][0] == 7



# ------------------------------------------------------------ the rejected modular prior
def test_mean_direction_prior_closed_forms_and_brute_force():
    """Table of negative gates, scoring family: s + lambda cos(V, dir)."""
    import math
    n, d = 9, 16
    # one-hot rows: dir = (1/n) sum e_i, cos(e_i, dir) = 1/sqrt(n)
    V = np.eye(d)[:n]
    out = O.score_mean_direction_prior(np.zeros(n), V, 2.0, 0.0)
    np.testing.assert_allclose(out, 2.0 / math.sqrt(n), rtol=1e-14)
    # identical rows: cosine 1 (up to eps); the base score passes through
    V = np.tile(np.arange(1.0, d + 1), (n, 1))
    s = np.linspace(-1, 1, n)
    np.testing.assert_allclose(O.score_mean_direction_prior(s, V, 0.5, 0.0), s + 0.5, rtol=1e-14)
    # rows cancelling in pairs: dir = 0, the eps keeps the term finite and zero
    V = np.concatenate([np.ones((4, d)), -np.ones((4, d))])
    np.testing.assert_array_equal(O.score_mean_direction_prior(np.ones(8), V, 3.0, 1e-6), np.ones(8))
    # a row opposite to the mean gets the negative sign; scaling a row does not change its cosine
    V = np.array([[1.0, 0.0], [1.0, 0.0], [1.0, 0.0], [-1.0, 0.0], [7.0, 0.0]])
    out = O.score_mean_direction_prior(np.zeros(5), V, 1.0, 0.0)
    np.testing.assert_allclose(out, [1, 1, 1, -1, 1], rtol=1e-14)
    # brute force with plain loops
    rng = np.random.default_rng(3)
    V = rng.normal(size=(7, 5)); s = rng.normal(size=7); eps = 1e-3
    dirv = [sum(V[j][e] for j in range(7)) / 7 for e in range(5)]
    nd = math.sqrt(sum(x * x for x in dirv))
    for i in range(7):
        dot = sum(V[i][e] * dirv[e] for e in range(5))
        ni = math.sqrt(sum(V[i][e] ** 2 for e in range(5)))
        want = s[i] + 0.7 * dot / ((ni + eps) * (nd + eps))
        assert abs(O.score_mean_direction_prior(s, V, 0.7, eps)[i] - want) < 1e-13


# ------------------------------------------------------------ score pooling
def test_score_pooling_matches_the_library_pooling_and_hand_values():
    """The smoothing step of observation-window scorers (Sec. 2's scorer family)."""
    import torch
    import torch.nn.functional as F
    s = np.array([1.0, 5.0, 2.0, 0.0, -3.0, 4.0])
    assert O.score_pool(s, 3).tolist() == [5, 5, 5, 2, 4, 4]
    np.testing.assert_allclose(O.score_pool(s, 3, mean=True), [2, 8 / 3, 7 / 3, -1 / 3, 1 / 3, 1 / 3], rtol=1e-15)
    assert O.score_pool(s, 1).tolist() == s.tolist() and O.score_pool(s, 1, mean=True).tolist() == s.tolist()
    assert O.score_pool(s, 63).tolist() == [5.0] * 6              # window wider than the row
    rng = np.random.default_rng(11)
    for n, k in [(1, 7), (9, 5), (40, 7), (100, 13), (33, 63)]:
        x = rng.normal(size=n)
        t = torch.from_numpy(x)[None, None]
        np.testing.assert_array_equal(O.score_pool(x, k), F.max_pool1d(t, k, stride=1, padding=k // 2)[0, 0].numpy())
        np.testing.assert_allclose(O.score_pool(x, k, mean=True),
                                   F.avg_pool1d(t, k, stride=1, padding=k // 2)[0, 0].numpy(), rtol=1e-12, atol=1e-15)


# ------------------------------------------------------------ randomized properties (hypothesis)
def _problem(draw_n, draw_seed):
    rng = np.random.default_rng(draw_seed)
    n = draw_n
    s = rng.normal(size=n).round(3)
    V = rng.normal(size=(n, 6))
    V[rng.integers(0, n)] = V[rng.integers(0, n)] * 2.0          # a pair of parallel rows now and then
    return s, V


def test_random_properties_of_algorithm1():
    """Facts that hold for every input (Sec. 4.1, Eq. 2-3): a token permutation permutes the picks
    (when no two gains tie), adding a constant to every score changes no pick and shifts every gain,
    the first pick is the argmax of s, and a larger budget only appends picks."""
    from hypothesis import given, settings, strategies as st

    @settings(max_examples=60, deadline=None)
    @given(n=st.integers(2, 24), seed=st.integers(0, 10**6), lam=st.sampled_from([0.0, 0.1, 0.5, 2.0]),
           kfrac=st.floats(0.1, 1.0))
    def run(n, seed, lam, kfrac):
        s, V = _problem(n, seed)
        k = max(1, int(round(kfrac * n)))
        r = O.alpha_select(s, V, k, lam)
        order, gain = r["order"], r["gain"]
        assert order[0] == int(np.flatnonzero(s == s.max())[0])
        assert len(set(order.tolist())) == k and np.all(np.diff(gain) <= 1e-12)
        # a larger budget appends
        if k < n:
            r2 = O.alpha_select(s, V, k + 1, lam)
            assert r2["order"][:k].tolist() == order.tolist()
        # constant shift of the scores
        r3 = O.alpha_select(s + 3.25, V, k, lam)
        assert r3["order"].tolist() == order.tolist()
        np.testing.assert_allclose(r3["gain"], gain + 3.25, rtol=0, atol=1e-9)
        # permutation equivariance, checked only when the run has no (near-)ties
        free = O.alpha_select(s, V, k, lam)
        if "second" in free and np.all(free["gain"] - free["second"] > 1e-9):
            perm = np.random.default_rng(seed + 1).permutation(n)
            rp = O.alpha_select(s[perm], V[perm], k, lam)
            assert perm[rp["order"]].tolist() == order.tolist()

    run()


def test_random_properties_of_the_budgeted_frame_and_the_epilogues():
    from hypothesis import given, settings, strategies as st

    @settings(max_examples=40, deadline=None)
    @given(n=st.integers(3, 20), seed=st.integers(0, 10**6), lam=st.sampled_from([0.1, 0.5, 2.0]))
    def run(n, seed, lam):
        s, V = _problem(n, seed)
        rng = np.random.default_rng(seed + 7)
        n_h = int(rng.integers(2, n + 1))
        b_h = int(rng.integers(1, n_h + 1))
        keep = np.zeros(n, dtype=bool)
        keep[rng.choice(n_h, size=int(rng.integers(0, b_h + 1)), replace=False)] = True
        r = O.select_budgeted(s, V, n_h, b_h, keep, lam)
        chosen = r["sorted"].tolist()
        assert len(chosen) == b_h and max(chosen) < n_h and set(np.flatnonzero(keep).tolist()) <= set(chosen)
        # every non-protected pick is the argmax of Eq. 2 over the free candidates, given everything before it
        Vh = O.signatures(V[:n_h], 1e-6)
        S = r["protected"].tolist()
        for i, g in zip(r["order"].tolist(), r["gain"].tolist()):
            gains = O.marginal_gains(s[:n_h], Vh, S, lam)
            gains[S] = -np.inf
            assert i == int(np.flatnonzero(gains == gains.max())[0]) and abs(gains[i] - g) < 1e-12
            S.append(i)
        # pooling: max-pool dominates the scores, mean-pool preserves the sum up to the zero padding at the ends
        k = int(rng.choice([1, 3, 5]))
        assert np.all(O.score_pool(s, k) >= s)
        inner = O.score_pool(np.pad(s, (k // 2, k // 2)), k, mean=True)
        np.testing.assert_allclose(inner.sum(), s.sum(), rtol=0, atol=1e-9)
        # the modular prior is bounded by |lambda_p| and vanishes with it
        pr = O.score_mean_direction_prior(s, V, 0.7, 1e-6) - s
        assert np.all(np.abs(pr) <= 0.7 + 1e-12)
        np.testing.assert_array_equal(O.score_mean_direction_prior(s, V, 0.0, 1e-6), s)

    run()
