"""Pins for the oracle's conformal layer: what the paper and the mathematics fix.

Each test is chosen so that a plausible slip in oracle/atts_oracle.py (wrong comparison
direction, strict vs inclusive ties, missing +1, off-by-one in the order statistic,
p < alpha instead of p <= alpha) fails at least one of them.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import atts_oracle as O
from synth import lognormal_scores

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "pvalue_ties.txt")


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


def test_golden_ties_fixture():
    """Hand-counted example following the tie formula in the proof of Proposition 1."""
    g = _read_golden()
    cal = np.array(g["cal"], dtype=np.float64)
    test = np.array(g["test"], dtype=np.float64)
    n = len(cal)
    c = O.rank_counts(cal, test)
    assert (c + 1).tolist() == [int(x) for x in g["pnum"]]
    assert n + 1 == int(g["pden"][0])
    p = O.p_values(c, n)
    assert np.allclose(p, np.array(g["pnum"], dtype=float) / float(g["pden"][0]), rtol=0, atol=1e-15)
    alphas = [float(a) for a in g["alpha"]]
    r = O.reject_ranks(alphas, n)
    assert r.tolist() == [int(x) for x in g["r"]]
    assert O.classify(c, r).tolist() == [int(x) for x in g["class"]]
    assert O.quantile_thresholds(cal, r).tolist() == [float(x) for x in g["quant"]]
    assert [n + 1 - int(x) for x in g["r"]] == [int(x) for x in g["kth"]]


def test_tie_formula_of_proposition_1_proof():
    """p = (sum_{l <= i} n_l) / (nm + 1) for pooled values sorted ascending, in the
    proof's own orientation (indicator  s_cal <= s_test); our nonconformity orientation
    is its mirror image under s -> -s."""
    rng = np.random.default_rng(7)
    for _ in range(50):
        pooled = rng.integers(0, 6, size=rng.integers(2, 12)).astype(np.float64)
        for i_test in range(len(pooled)):
            test = pooled[i_test]
            cal = np.delete(pooled, i_test)
            vals, mult = np.unique(pooled, return_counts=True)
            i = int(np.searchsorted(vals, test))
            expect = Fraction(int(mult[: i + 1].sum()), len(pooled))
            # mirror: the proof counts s_cal <= s_test; negate both to use our >= count
            c = O.rank_counts(-cal, np.array([-test]))[0]
            assert Fraction(int(c) + 1, len(cal) + 1) == expect


def test_distinct_scores_give_uniform_p_values():
    """Proposition 1: distinct scores => p ~ U{1/(N+1), ..., 1}.  Exact enumeration: let
    the test point be each of the N+1 pooled values in turn."""
    rng = np.random.default_rng(3)
    for n in (1, 2, 7, 40):
        pooled = rng.permutation(np.arange(n + 1, dtype=np.float64) * 0.37 - 2.0)
        got = []
        for i in range(n + 1):
            c = O.rank_counts(np.delete(pooled, i), pooled[i:i + 1])[0]
            got.append(int(c) + 1)
        assert sorted(got) == list(range(1, n + 2))
        # largest score is the least conforming: smallest p
        i_max = int(np.argmax(pooled))
        assert O.rank_counts(np.delete(pooled, i_max), pooled[i_max:i_max + 1])[0] == 0


@pytest.mark.parametrize("alpha", [0.05, 0.1, 0.25, 0.4, 0.5, 0.9])
def test_validity_exact_enumeration(alpha):
    """P(p <= alpha) = floor(alpha (N+1)) / (N+1) <= alpha for distinct scores (the case
    split at the end of Proposition 1's proof), and <= that with ties."""
    rng = np.random.default_rng(11)
    for n in (3, 9, 19, 57):
        for ties in (False, True):
            pooled = (rng.integers(0, max(2, n // 3), n + 1).astype(float) if ties
                      else rng.permutation(n + 1).astype(float))
            rejected = 0
            for i in range(n + 1):
                cal = np.delete(pooled, i)
                c = O.rank_counts(cal, pooled[i:i + 1])
                rejected += int(O.classify(c, O.reject_ranks([alpha], n))[0])
            bound = math.floor(Fraction(alpha).limit_denominator(1000) * (n + 1))
            if ties:
                assert rejected <= bound
            else:
                assert rejected == bound
            assert Fraction(rejected, n + 1) <= Fraction(alpha).limit_denominator(1000)


def test_monte_carlo_coverage_and_takeover_rate():
    """Theorem 1: accept rate >= 1 - alpha on exchangeable scores; the measured take-over
    rate sits at alpha (the paper's budget-prediction figure reports 25.1-30.5 % at
    alpha = 0.25)."""
    alpha, n, m = 0.25, 999, 20000
    s = lognormal_scores(n + m, seed=1234).astype(np.float64)
    cal, test = s[:n], s[n:]
    c = O.rank_counts_sorted(cal, test)
    rej = O.classify(c, O.reject_ranks([alpha], n)).mean()
    sigma = math.sqrt(alpha * (1 - alpha) / m)
    assert 1.0 - rej >= 1.0 - alpha - 5 * sigma
    assert abs(rej - alpha) < 0.02


def test_closed_forms_extremes_and_direction():
    cal = np.array([3.0, -1.0, 2.5, 0.0, 7.0])
    c = O.rank_counts(cal, np.array([8.0, 7.0, -1.0, -5.0, 2.5]))
    assert c.tolist() == [0, 1, 5, 5, 3]          # inclusive ties; larger score -> fewer
    p = O.p_values(c, len(cal))
    assert p[0] == 1.0 / 6.0 and p[3] == 1.0


def test_ieee_special_values():
    cal = np.array([np.nan, -0.0, 0.0, np.inf, -np.inf, 1.0])
    test = np.array([0.0, -0.0, np.nan, np.inf, -np.inf])
    c = O.rank_counts(cal, test)
    assert c.tolist() == [4, 4, 0, 1, 5]
    assert O.rank_counts_sorted(cal, test).tolist() == c.tolist()
    # NaN test score -> c = 0 -> smallest p -> rejected at every level with r >= 1
    assert O.classify(c[2:3], np.array([1, 3]))[0] == 2


def test_brute_force_equals_sorted_rank():
    rng = np.random.default_rng(5)
    for n, m in ((1, 5), (17, 33), (1000, 257), (4096, 300)):
        cal = np.round(rng.lognormal(size=n), 2)      # rounding makes ties
        test = np.round(rng.lognormal(size=m), 2)
        assert np.array_equal(O.rank_counts(cal, test), O.rank_counts_sorted(cal, test))


def test_reject_ranks_at_the_published_workload_sizes():
    got = [int(O.reject_ranks([a], n)[0]) for a, n in
           ((0.1, 200), (0.1, 1000), (0.05, 5000), (0.1, 2000), (0.05, 1 << 20), (0.2, 1 << 20))]
    exact = [math.floor(Fraction(a).limit_denominator(100) * (n + 1)) for a, n in
             ((0.1, 200), (0.1, 1000), (0.05, 5000), (0.1, 2000), (0.05, 1 << 20), (0.2, 1 << 20))]
    assert got == exact == [20, 100, 250, 200, 52428, 209715]


def test_integer_rule_equals_p_le_alpha_in_exact_arithmetic():
    for n in (1, 4, 9, 99, 200):
        for a in (Fraction(1, 10), Fraction(1, 4), Fraction(2, 5), Fraction(1, 2), Fraction(19, 20)):
            r = int(O.reject_ranks([float(a)], n)[0])
            if (a * (n + 1)).denominator == 1:
                # exactly on an integer boundary the binary64 product may land on either
                # side; the rule is then defined by the binary64 product
                assert abs(r - a * (n + 1)) <= 1
                continue
            for c in range(n + 1):
                assert (c + 1 <= r) == (Fraction(c + 1, n + 1) <= a)


def test_class_monotone_in_score_and_level_collapse():
    cal = lognormal_scores(500, seed=9).astype(np.float64)
    test = np.sort(lognormal_scores(300, seed=10).astype(np.float64))
    c = O.rank_counts(cal, test)
    assert np.all(np.diff(c) <= 0)
    cls = O.classify(c, O.reject_ranks([0.05, 0.2], 500))
    assert np.all(np.diff(cls.astype(int)) >= 0)
    assert set(cls.tolist()) == {0, 1, 2}
    p = O.p_values(c, 500)
    assert (cls == 2).sum() == (p <= 0.05).sum() and (cls >= 1).sum() == (p <= 0.2).sum()
    same = O.classify(c, O.reject_ranks([0.2, 0.2], 500))
    assert set(same.tolist()) <= {0, 2} and np.array_equal(same >= 1, cls >= 1)


def test_quantile_identity_exhaustive_small():
    """c + 1 <= r  <=>  s > Q  for every multiset over a small alphabet, every r, every s."""
    alphabet = [0.0, 1.0, 2.0]
    probes = np.array([-1.0, 0.0, 0.5, 1.0, 1.5, 2.0, 3.0])
    for n in (1, 2, 3, 4):
        for cal in itertools.combinations_with_replacement(alphabet, n):
            cal = np.array(cal)
            c = O.rank_counts(cal, probes)
            for r in range(0, n + 2):
                q = O.quantile_thresholds(cal, np.array([r]))[0]
                assert np.array_equal(c + 1 <= r, probes > q), (cal, r, q)


def test_quantile_is_the_classic_order_statistic():
    """Eq. "quantile": tau is the ceil((N+1)(1-alpha))-th smallest score."""
    cal = lognormal_scores(999, seed=21).astype(np.float64)
    srt = np.sort(cal)
    for a in (Fraction(1, 20), Fraction(1, 10), Fraction(1, 4), Fraction(2, 5)):
        kth = math.ceil((len(cal) + 1) * (1 - a))
        q = O.quantile_thresholds(cal, O.reject_ranks([float(a)], len(cal)))[0]
        assert q == srt[kth - 1]
    assert O.quantile_thresholds(cal, np.array([0]))[0] == np.inf
    assert O.quantile_thresholds(cal, np.array([len(cal) + 1]))[0] == -np.inf


def test_online_append_is_multiset_union():
    s = lognormal_scores(700, seed=33).astype(np.float64)
    test = lognormal_scores(64, seed=34).astype(np.float64)
    cs = O.CalibrationSet()
    for lo, hi in ((0, 200), (200, 201), (201, 201), (201, 700)):
        cs.append(s[lo:hi])
        c, p, cls, q = cs.classify(test, [0.1, 0.3])
        assert len(cs) == hi
        assert np.array_equal(c, O.rank_counts(s[:hi], test))
        assert np.array_equal(cls, O.classify(c, O.reject_ranks([0.1, 0.3], hi)))
    perm = np.random.default_rng(0).permutation(700)
    assert np.array_equal(O.rank_counts(s[perm], test), c)     # order-free


def test_score_modes():
    lp = -np.abs(np.random.default_rng(1).normal(size=37))
    assert math.isclose(O.conformity_score(lp, O.SUM_NLL), 37 * O.conformity_score(lp, O.MEAN_NLL))
    assert O.conformity_score(lp, O.MEAN_NLL) > 0          # NLL: larger = less conforming
    assert math.isclose(O.conformity_score(lp, O.SUM_NLL), -math.fsum(lp))


# ---- conditional coverage (Proposition 2): every input ranked against its own calibration scores --------

def _read_conditional_fixture():
    alphas, inputs, cur = None, [], None
    for line in open(os.path.join(os.path.dirname(GOLDEN), "conditional_small.txt")).read().splitlines():
        line = line.split("#")[0].strip()
        if not line:
            continue
        key, *vals = line.split()
        if key == "alpha":
            alphas = [float(v) for v in vals]
        elif key == "cal":
            cur = {"cal": [float(v) for v in vals]}
            inputs.append(cur)
        elif key == "pden":
            cur[key] = int(vals[0])
        elif key == "test":
            cur[key] = [float(v) for v in vals]
        else:
            cur[key] = [int(v) for v in vals]
    return alphas, inputs


def test_conditional_golden_fixture():
    alphas, inputs = _read_conditional_fixture()
    c, p, cls = O.conditional_classify([i["cal"] for i in inputs], [i["test"] for i in inputs], alphas)
    for k, i in enumerate(inputs):
        assert c[k].tolist() == i["count"], k
        assert cls[k].tolist() == i["class"], k
        assert np.array_equal(p[k], np.array(i["pnum"], dtype=np.float64) / i["pden"]), k


def test_conditional_uniform_law_by_enumeration():
    """Proposition 2: with m distinct calibration scores of the input and one candidate, all exchangeable, the
    candidate's p-value is uniform on {1/(m+1), ..., 1}: enumerate every ordering of m + 1 distinct values and
    let each position be the candidate once."""
    import itertools
    for m in (1, 2, 4, 5):
        vals = np.arange(1.0, m + 2.0)
        hist = np.zeros(m + 2, dtype=np.int64)
        for perm in itertools.permutations(vals):
            c, p, _ = O.conditional_classify([perm[:m]], [[perm[m]]], [0.5])
            hist[int(c[0][0]) + 1] += 1
            assert p[0][0] == (c[0][0] + 1) / (m + 1)
        assert hist[0] == 0 and len(set(hist[1:])) == 1                    # every value k/(m+1) equally often
        for alpha in (0.1, 0.34, 0.5, 0.8):                               # hence P(p <= alpha) = floor(alpha(m+1))/(m+1) <= alpha
            rej = sum(hist[k] for k in range(1, m + 2) if k / (m + 1) <= alpha) / hist.sum()
            assert rej == math.floor(alpha * (m + 1)) / (m + 1) <= alpha


def test_conditional_is_the_marginal_rule_per_input_and_inputs_do_not_interact():
    rng = np.random.default_rng(5)
    cal = [np.round(rng.lognormal(size=n), 1) for n in (0, 1, 16, 33, 128)]
    test = [np.round(rng.lognormal(size=n), 1) for n in (3, 0, 16, 64, 7)]
    alphas = [0.05, 0.2, 0.2, 0.7]
    c, p, cls = O.conditional_classify(cal, test, alphas)
    for k in range(len(cal)):
        ck = O.rank_counts_sorted(cal[k], test[k]) if len(cal[k]) else np.zeros(len(test[k]), dtype=np.int64)
        assert np.array_equal(c[k], ck)
        assert np.array_equal(cls[k], O.classify(ck, O.reject_ranks(alphas, len(cal[k]))))
        assert np.array_equal(p[k], O.p_values(ck, len(cal[k])))
    order = [3, 0, 4, 2, 1]
    c2, p2, cls2 = O.conditional_classify([cal[i] for i in order], [test[i] for i in order], alphas)
    for pos, i in enumerate(order):
        assert np.array_equal(c2[pos], c[i]) and np.array_equal(cls2[pos], cls[i])
    # pooling the inputs (the marginal rule) gives different counts: the two notions really differ
    pooled = O.rank_counts(np.concatenate(cal), test[3])
    assert not np.array_equal(pooled, c[3])
