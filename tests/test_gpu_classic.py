"""Parity of the classic (synchronous) pipeline -- atts_classic_normalize / _threshold / _prediction_sets -- with the
oracle: normalised scores within fp32 round-off of the fp64 ones; threshold and set membership bit-exact when both sides
are given the same fp32 normalised scores; the chained calls agree with the oracle's chain except on candidates whose
score lies within round-off of the threshold."""
import numpy as np
import pytest
import torch

from oracle import atts_oracle as O
from util import announce, dev, ws

pytestmark = pytest.mark.gpu

RTOL = 1e-5     # fp32 exp of a difference below 128 (4e-6) + fp32 sum and quotient


def _normalize(A, nll):
    s = torch.full(nll.shape, -5.0, dtype=torch.float32, device="cuda")
    A.atts_classic_normalize(dev(nll), s)
    torch.cuda.synchronize()
    return s.cpu().numpy()


@pytest.mark.parametrize("n,m", [(1, 1), (7, 3), (50, 16), (33, 64), (9, 65), (5, 100), (3, 1000), (4099, 16)])
def test_normalize_against_oracle(n, m):
    import paper_2509_15148_amd as A
    announce("classic normalize", n, m)
    rng = np.random.default_rng(100 * n + m)
    nll = rng.uniform(8.0, 14.0, size=(n, m)).astype(np.float32)          # mean-NLL scores near ln V
    got = _normalize(A, nll)
    want = O.classic_softmax_scores(nll.astype(np.float64))
    np.testing.assert_allclose(got, want, rtol=RTOL, atol=1e-30)
    np.testing.assert_allclose(got.sum(axis=1), 1.0, rtol=1e-5)
    # sum-NLL scores of long drafts: thousands, shares of all but the best few candidates underflow to 0
    big = rng.uniform(2000.0, 2040.0, size=(n, m)).astype(np.float32)
    got = _normalize(A, big)
    want = O.classic_softmax_scores(big.astype(np.float64))
    np.testing.assert_allclose(got, want, rtol=RTOL, atol=1e-37)
    assert np.isfinite(got).all()


def _threshold(A, s32, alpha):
    tau = torch.full((1,), -3.0, dtype=torch.float32, device="cuda")
    A.atts_classic_threshold(dev(s32), alpha, tau, ws(A.atts_classic_workspace_bytes(len(s32))))
    torch.cuda.synchronize()
    return tau


@pytest.mark.parametrize("N", [1, 9, 1000, 8192 * 3 + 5, 65536, 65537, 300001])
def test_threshold_and_sets_bit_exact(N):
    """Same fp32 normalised scores on both sides: tau is a stored score and membership an IEEE comparison."""
    import paper_2509_15148_amd as A
    announce("classic threshold", N)
    rng = np.random.default_rng(N)
    m = 16
    n_in = -(-N // m)
    s32 = O.classic_softmax_scores(rng.uniform(8.0, 14.0, size=(n_in, m))).astype(np.float32).ravel()[:N].copy()
    if N > 4:
        s32[N // 2] = s32[0]                                               # ties
        s32[N // 3] = s32[1]
    test = np.concatenate([s32[: min(N, 4096)], rng.uniform(0, 1, size=1000).astype(np.float32),
                           np.array([np.nan, 0.0, 1.0, np.inf], dtype=np.float32)])
    for alpha in (0.001, 0.05, 0.1, 0.2, 0.5, 0.999):
        tau = _threshold(A, s32, alpha)
        want = O.classic_threshold(s32.astype(np.float64), alpha)
        got = float(tau.cpu().numpy()[0])
        assert got == np.float32(want), (N, alpha, got, want)
        member = torch.full((len(test),), 9, dtype=torch.uint8, device="cuda")
        A.atts_classic_prediction_sets(dev(test), tau, member)
        torch.cuda.synchronize()
        assert np.array_equal(member.cpu().numpy(), O.classic_prediction_sets(test.astype(np.float64), want))


def test_chain_against_oracle():
    """nll -> normalise -> global threshold -> sets, all on the device, against the oracle's fp64 chain."""
    import paper_2509_15148_amd as A
    announce("classic chain")
    rng = np.random.default_rng(2024)
    n_cal, n_test, m, alpha = 4000, 500, 16, 0.1
    cal = rng.normal(11.9, 0.4, size=(n_cal, m)).astype(np.float32)
    test = rng.normal(11.9, 0.4, size=(n_test, m)).astype(np.float32)
    s_cal = torch.empty(n_cal, m, dtype=torch.float32, device="cuda")
    s_test = torch.empty(n_test, m, dtype=torch.float32, device="cuda")
    tau = torch.empty(1, dtype=torch.float32, device="cuda")
    member = torch.empty(n_test, m, dtype=torch.uint8, device="cuda")
    A.atts_classic_normalize(dev(cal), s_cal)
    A.atts_classic_normalize(dev(test), s_test)
    A.atts_classic_threshold(s_cal.view(-1), alpha, tau, ws(A.atts_classic_workspace_bytes(n_cal * m)))
    A.atts_classic_prediction_sets(s_test.view(-1), tau, member.view(-1))
    torch.cuda.synchronize()
    o_cal = O.classic_softmax_scores(cal.astype(np.float64))
    o_test = O.classic_softmax_scores(test.astype(np.float64))
    o_tau = O.classic_threshold(o_cal, alpha)
    o_mem = O.classic_prediction_sets(o_test, o_tau)
    assert float(tau.cpu()[0]) == pytest.approx(o_tau, rel=RTOL)
    got = member.cpu().numpy()
    differ = got != o_mem
    # a differing decision must be a close call: the oracle's score within round-off of its threshold
    assert (np.abs(o_test[differ] - o_tau) <= 2 * RTOL * o_tau).all()
    assert differ.mean() < 1e-3
    # about alpha of the candidates are members (exchangeable test and calibration data)
    assert abs(got.mean() - alpha) < 0.02
