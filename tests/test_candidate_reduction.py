"""Properties of Algorithm 1 (paper Sec. 4.1, Eq. 2-3) that the HIP path relies on when it
shrinks the candidate set of a head before running the pick chain.  Checked on the fp64
oracle; CPU only."""
import numpy as np
import pytest

from oracle import alpha_oracle as O


def _case(seed, n, d=16, spread=1.0):
    rng = np.random.default_rng(seed)
    centres = rng.normal(size=(6, d))
    V = centres[rng.integers(0, 6, size=n)] + 0.2 * rng.normal(size=(n, d))
    s = np.exp(spread * rng.normal(size=n))
    return s, V


@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("lam", [0.05, 0.5, 1.0])
def test_tokens_below_the_score_bound_are_never_picked(seed, lam):
    # a cosine is at most 1, so one of the k best-scored tokens always offers a gain of at
    # least s_(k) - lambda; a token with s_j below that can never be the argmax of Eq. 3
    n, k = 60, 20
    s, V = _case(seed, n)
    r = O.alpha_select(s, V, k, lam, 1e-6)
    s_k = np.sort(s)[::-1][k - 1]
    assert np.all(s[r["order"]] >= s_k - lam)
    assert np.all(r["gain"] >= s_k - lam - 1e-12)


@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("lam", [0.05, 0.5, 1.0])
def test_selection_on_the_survivors_equals_selection_on_the_head(seed, lam):
    # dropping the tokens below the bound (survivors keep their order) changes nothing
    n, k = 60, 20
    s, V = _case(seed, n)
    full = O.alpha_select(s, V, k, lam, 1e-6)
    s_k = np.sort(s)[::-1][k - 1]
    keep = np.flatnonzero(s >= s_k - lam)
    red = O.alpha_select(s[keep], V[keep], k, lam, 1e-6)
    np.testing.assert_array_equal(keep[red["order"]], full["order"])
    np.testing.assert_allclose(red["gain"], full["gain"], rtol=0, atol=1e-12)


def test_cut_at_the_best_scores_is_valid_when_it_stays_below_every_gain():
    # keep only the M best-scored tokens; if the best score left out is below the smallest
    # pick gain of the run on the kept tokens, that run is the run on the whole head (a
    # left-out token's gain never exceeds its score, pick gains never increase).  The
    # condition must hold in some cases and fail in others, so that the check is not vacuous.
    n, k, lam = 80, 16, 0.3
    outcomes = []
    for seed in range(12):
        s, V = _case(seed, n, spread=0.6)
        full = O.alpha_select(s, V, k, lam, 1e-6)
        for M in (k, k + 4, k + 12, 40):
            keep = np.sort(np.argsort(-s, kind="stable")[:M])
            left_out = np.setdiff1d(np.arange(n), keep)
            red = O.alpha_select(s[keep], V[keep], k, lam, 1e-6)
            ok = s[left_out].max() < red["gain"].min()
            outcomes.append(ok)
            if ok:
                np.testing.assert_array_equal(keep[red["order"]], full["order"])
    assert any(outcomes) and not all(outcomes)


def test_pick_gains_never_increase():
    for seed in range(6):
        s, V = _case(seed, 50)
        g = O.alpha_select(s, V, 30, 0.7, 1e-6)["gain"]
        assert np.all(np.diff(g) <= 1e-12)
