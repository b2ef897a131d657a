"""Parity of atts_classify_conditional with the oracle: ranks and classes bit-exact, p-values equal to the
oracle's binary64 p rounded once to fp32 (conditional coverage, Proposition 2)."""
import os

import numpy as np
import pytest
import torch

from oracle import atts_oracle as O
from synth import lognormal_scores
from util import announce, dev

pytestmark = pytest.mark.gpu


def _run(A, cal_sets, test_sets, alphas, want_p=True):
    cal_off = np.concatenate([[0], np.cumsum([len(c) for c in cal_sets])]).astype(np.int64)
    test_off = np.concatenate([[0], np.cumsum([len(t) for t in test_sets])]).astype(np.int64)
    cal = np.concatenate([np.asarray(c, np.float32) for c in cal_sets] + [np.zeros(0, np.float32)])
    test = np.concatenate([np.asarray(t, np.float32) for t in test_sets] + [np.zeros(0, np.float32)])
    M = len(test)
    ranks = torch.full((M,), -7, dtype=torch.int32, device="cuda")
    cls = torch.full((M,), 99, dtype=torch.uint8, device="cuda")
    p = torch.full((M,), -1.0, dtype=torch.float32, device="cuda") if want_p else None
    A.atts_classify_conditional(dev(cal), dev(cal_off), dev(test), dev(test_off), alphas, ranks, p, cls)
    torch.cuda.synchronize()
    return ranks.cpu().numpy(), cls.cpu().numpy(), None if p is None else p.cpu().numpy(), test_off


def _check(A, cal_sets, test_sets, alphas):
    ranks, cls, p, off = _run(A, cal_sets, test_sets, alphas)
    c_ref, p_ref, cls_ref = O.conditional_classify([np.asarray(c, np.float32) for c in cal_sets],
                                                   [np.asarray(t, np.float32) for t in test_sets], alphas)
    for x in range(len(cal_sets)):
        sl = slice(off[x], off[x + 1])
        assert np.array_equal(ranks[sl].astype(np.int64), c_ref[x]), x
        assert np.array_equal(cls[sl], cls_ref[x]), x
        assert np.array_equal(p[sl], p_ref[x].astype(np.float32)), x
    return ranks, cls


def test_golden_fixture_and_special_values():
    import paper_2509_15148_amd as A
    announce("conditional golden")
    from test_oracle_conformal import _read_conditional_fixture
    alphas, inputs = _read_conditional_fixture()
    ranks, cls = _check(A, [i["cal"] for i in inputs], [i["test"] for i in inputs], alphas)
    assert ranks.tolist() == sum((i["count"] for i in inputs), [])
    special = np.array([0.5, -0.0, 0.0, np.inf, -np.inf, np.nan, 1e-45, -1e-45, 2.0, 2.0], np.float32)
    probes = np.array([0.0, -0.0, np.nan, np.inf, -np.inf, 1e-45, -1e-45, 2.0, 1.0], np.float32)
    _check(A, [special, special[:3]], [probes, probes], [0.3, 0.75])


@pytest.mark.parametrize("seed", [1, 2])
def test_ragged_inputs_against_the_oracle(seed):
    """Empty inputs, inputs without candidates, sets below / at / above one 64-lane block, many ties."""
    import paper_2509_15148_amd as A
    announce("conditional ragged", seed)
    rng = np.random.default_rng(seed)
    m_sizes = [0, 1, 63, 64, 65, 128, 200, 1000, 5, 0, 16, 4097]
    k_sizes = [4, 0, 64, 65, 1, 130, 16, 300, 0, 0, 16, 70]
    cal = [np.round(rng.lognormal(size=m), 2).astype(np.float32) for m in m_sizes]
    test = [np.round(rng.lognormal(size=k), 2).astype(np.float32) for k in k_sizes]
    for alphas in ([0.25], [0.05, 0.2], [0.01, 0.3, 0.3, 0.9]):
        _check(A, cal, test, alphas)
    # scores only: no p-values requested
    r1, c1, p1, _ = _run(A, cal, test, [0.05, 0.2], want_p=False)
    r2, c2 = _check(A, cal, test, [0.05, 0.2])
    assert p1 is None and np.array_equal(r1, r2) and np.array_equal(c1, c2)


def test_many_small_inputs():
    """4096 inputs x 64 own calibration scores x 64 candidates (the batch shape bench.py times); the reject
    fraction per level is close to alpha (budget control per input, Sec. "Budget Prediction")."""
    import paper_2509_15148_amd as A
    S, m, k = 4096, 64, 64
    announce("conditional many", S, m, k)
    cal = lognormal_scores(S * m, seed=31).reshape(S, m)
    test = lognormal_scores(S * k, seed=32).reshape(S, k)
    ranks, cls = _check(A, list(cal), list(test), [0.05, 0.2])
    frac = np.bincount(cls, minlength=3) / cls.size
    assert abs(frac[2] - 3 / 65) < 0.005 and abs(frac[1] + frac[2] - 13 / 65) < 0.01   # floor(alpha 65) / 65


def test_argument_errors():
    import paper_2509_15148_amd as A
    announce("conditional errors")
    off = dev(np.array([0, 2], np.int64))
    x = dev(np.array([1.0, 2.0], np.float32))
    r = torch.empty(2, dtype=torch.int32, device="cuda")
    c = torch.empty(2, dtype=torch.uint8, device="cuda")
    for bad in ([], [0.0], [1.0], [0.3, 0.2], [0.1] * 9, [float("nan")]):
        with pytest.raises(A.AttsError) as e:
            A.atts_classify_conditional(x, off, x, off, bad, r, None, c)
        assert e.value.code == A.ERR_INVALID_ARG
    with pytest.raises(A.AttsError):
        A.atts_classify_conditional(x, off, x, dev(np.array([0, 1, 2], np.int64)), [0.1], r, None, c)
    # no inputs at all is a no-op
    z = dev(np.array([0], np.int64))
    A.atts_classify_conditional(x[:0], z, x[:0], z, [0.1], r[:0], None, c[:0])
