"""Pins for the oracle's classic (synchronous) pipeline: Sec. "Preliminary", Eq. "softmax", Eq. "quantile",
Eq. "pred_set".  Chosen so that a slip (softmax of +l instead of -l, normalising over the wrong axis, an off-by-one
order statistic, ">" instead of ">=") fails at least one of them.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import atts_oracle as O
from synth import lognormal_scores

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "classic_small.txt")


def _read_golden():
    rows = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            rows[key] = vals
    return rows


def test_golden_classic_fixture():
    g = _read_golden()
    e = np.array([Fraction(int(a), int(b)) for a, b in zip(g["exp_neg_l_num"], g["exp_neg_l_den"])], dtype=object).reshape(3, 3)
    nll = np.array([[-math.log(float(x)) for x in row] for row in e])
    s = O.classic_softmax_scores(nll)
    want = np.array([float(Fraction(int(a), int(b))) for a, b in zip(g["s_num"], g["s_den"])]).reshape(3, 3)
    np.testing.assert_allclose(s, want, rtol=1e-14)
    for i, alpha in enumerate(g["alpha"]):
        tau = O.classic_threshold(s, float(alpha))
        assert tau == pytest.approx(float(Fraction(int(g["tau_num"][i]), int(g["tau_den"][i]))), rel=1e-14)
        members = O.classic_prediction_sets(s, tau)
        assert members.dtype == np.uint8
        assert members.ravel().tolist() == [int(x) for x in g[f"members_{i}"]]


def test_softmax_rows_sum_to_one_and_shift_invariance():
    rng = np.random.default_rng(7)
    nll = rng.uniform(0.0, 30.0, size=(50, 16))
    s = O.classic_softmax_scores(nll)
    np.testing.assert_allclose(s.sum(axis=1), 1.0, rtol=1e-14)
    assert (s > 0).all()
    # a constant added to every loss of an input cancels in the quotient
    s2 = O.classic_softmax_scores(nll + rng.uniform(0, 5, size=(50, 1)))
    np.testing.assert_allclose(s2, s, rtol=1e-12)
    # the normalisation runs over the candidates of ONE input: rows are independent
    s3 = O.classic_softmax_scores(nll[3:4])
    np.testing.assert_allclose(s3[0], s[3], rtol=1e-14)
    # the smaller loss gets the larger share (softmax of -l, not of +l)
    assert (np.argmax(s, axis=1) == np.argmin(nll, axis=1)).all()


def test_softmax_two_candidates_is_the_logistic_function():
    d = np.linspace(-20, 20, 41)
    nll = np.stack([np.full_like(d, 5.0), 5.0 + d], axis=1)       # l_1 - l_0 = d
    s = O.classic_softmax_scores(nll)
    np.testing.assert_allclose(s[:, 0], 1.0 / (1.0 + np.exp(-d)), rtol=1e-13)
    assert O.classic_softmax_scores(np.array([[3.7]]))[0, 0] == 1.0           # m = 1


def test_softmax_large_sum_scores_do_not_underflow():
    nll = np.array([[3000.0, 3000.0 + math.log(3.0)]])            # shares 3/4 and 1/4
    np.testing.assert_allclose(O.classic_softmax_scores(nll)[0], [0.75, 0.25], rtol=1e-12)


@pytest.mark.parametrize("n,alpha", [(9, 0.3), (200, 0.1), (1000, 0.1), (5000, 0.05), (2000, 0.1), (37, 0.5), (5, 0.9), (5, 0.05)])
def test_threshold_is_the_order_statistic_by_brute_force(n, alpha):
    s = lognormal_scores(n, 11 + n).astype(np.float64)
    s[n // 2] = s[0]                                              # a tie
    tau = O.classic_threshold(s, alpha)
    k = math.ceil(Fraction(n + 1) * (1 - Fraction(alpha).limit_denominator(1000)))   # ceil((N + 1)(1 - alpha)), exact
    if k > n:
        assert tau == math.inf
        return
    # definition of the k-th smallest: the least value v of the set with #{s <= v} >= k
    cands = [v for v in s if np.count_nonzero(s <= v) >= k]
    assert tau == min(cands)
    assert np.count_nonzero(s < tau) < k <= np.count_nonzero(s <= tau)


def test_set_size_on_distinct_scores():
    """With N distinct scores, exactly floor(alpha (N + 1)) of them are >= tau: the set holds the top alpha share."""
    for n, alpha in [(999, 0.1), (4999, 0.05), (1999, 0.1), (200, 0.25)]:
        s = np.random.default_rng(n).permutation(n).astype(np.float64) / n
        tau = O.classic_threshold(s, alpha)
        members = O.classic_prediction_sets(s, tau)
        assert int(members.sum()) == math.floor(Fraction(alpha).limit_denominator(1000) * (n + 1))
        # inclusive: the threshold itself is a member
        assert members[np.argmax(s == tau)] == 1


def test_threshold_matches_the_rank_rule_quantile():
    """Same order statistic as the one the asynchronous rule's thresholds use (Eq. "quantile" is one equation)."""
    s = lognormal_scores(777, 5).astype(np.float64)
    for alpha in (0.05, 0.1, 0.2, 0.5):
        assert O.classic_threshold(s, alpha) == O.quantile_thresholds(s, O.reject_ranks([alpha], len(s)))[0]


def test_needs_all_m_scores():
    """The decision about one candidate changes with the OTHER candidates of its input (what makes the design
    synchronous), while its unnormalised score and p-value rank do not."""
    cal = O.classic_softmax_scores(np.random.default_rng(1).uniform(8, 14, size=(64, 8)))
    tau = O.classic_threshold(cal, 0.2)
    a = np.array([[10.0, 12.0, 12.0, 12.0, 12.0, 12.0, 12.0, 12.0]])
    b = np.array([[10.0, 8.0, 8.0, 8.0, 8.0, 8.0, 8.0, 8.0]])
    ma = O.classic_prediction_sets(O.classic_softmax_scores(a), tau)
    mb = O.classic_prediction_sets(O.classic_softmax_scores(b), tau)
    assert ma[0, 0] == 1 and mb[0, 0] == 0
