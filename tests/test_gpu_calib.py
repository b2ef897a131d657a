"""Parity of atts_calibrate_online / atts_classify_ordinal with the oracle: ranks, classes and
thresholds bit-exact, p-values equal to the oracle's binary64 p rounded once to fp32."""
import numpy as np
import pytest
import torch

from oracle import atts_oracle as O
from synth import WORKLOADS, lognormal_scores
from util import announce, dev

pytestmark = pytest.mark.gpu


def _classify(A, calib, test, alphas, want_p=True, want_q=True):
    M = len(test)
    t = dev(np.asarray(test, dtype=np.float32))
    ranks = torch.full((M,), -7, dtype=torch.int32, device="cuda")
    cls = torch.full((M,), 99, dtype=torch.uint8, device="cuda")
    p = torch.empty(M, dtype=torch.float32, device="cuda") if want_p else None
    q = torch.empty(len(alphas), dtype=torch.float32, device="cuda") if want_q else None
    A.atts_classify_ordinal(calib, t, alphas, ranks, p, cls, q)
    torch.cuda.synchronize()
    return (ranks.cpu().numpy(), cls.cpu().numpy(), None if p is None else p.cpu().numpy(),
            None if q is None else q.cpu().numpy())


def _check_against_oracle(A, calib, cal_np, test, alphas, brute=True):
    ranks, cls, p, q = _classify(A, calib, test, alphas)
    n = len(cal_np)
    c = (O.rank_counts if brute else O.rank_counts_sorted)(cal_np, test)
    r = O.reject_ranks(alphas, n)
    assert np.array_equal(ranks.astype(np.int64), c)
    assert np.array_equal(cls, O.classify(c, r))
    assert np.array_equal(p, O.p_values(c, n).astype(np.float32))
    assert np.array_equal(q, O.quantile_thresholds(cal_np, r).astype(np.float32), equal_nan=True)
    # decisions only (ranks = NULL): the threshold form of the same rule must give the same classes and thresholds
    M = len(test)
    cls2 = torch.full((M,), 77, dtype=torch.uint8, device="cuda")
    q2 = torch.empty(len(alphas), dtype=torch.float32, device="cuda")
    A.atts_classify_ordinal(calib, dev(np.asarray(test, dtype=np.float32)), alphas, None, None, cls2, q2)
    torch.cuda.synchronize()
    assert np.array_equal(cls2.cpu().numpy(), cls)
    assert np.array_equal(q2.cpu().numpy(), q, equal_nan=True)
    if M > 1:                                                  # pointers that are not 16- / 4-byte aligned
        t_all = dev(np.asarray(test, dtype=np.float32))
        cls3 = torch.full((M,), 77, dtype=torch.uint8, device="cuda")
        A.atts_classify_ordinal(calib, t_all[1:], alphas, None, None, cls3[1:], None)
        torch.cuda.synchronize()
        assert np.array_equal(cls3.cpu().numpy()[1:], cls[1:])
    return ranks, cls


def test_small_with_ties_and_special_values():
    import paper_2509_15148_amd as A
    announce("calib small/special")
    cal = np.array([0.5, 1.0, 1.0, 2.0, 2.0, 2.0, 3.5, 4.0, 4.0, -0.0, 0.0, np.inf, -np.inf, np.nan, 1e-45, -1e-45],
                   dtype=np.float32)
    test = np.array([2.0, 0.25, 5.0, 1.0, 3.75, 0.0, -0.0, np.nan, np.inf, -np.inf, 1e-45, -3.0], dtype=np.float32)
    c = A.Calib(64)
    A.atts_calibrate_online(c, dev(cal))
    assert A.atts_calib_size(c) == len(cal)
    for alphas in ([0.3], [0.3, 0.75], [0.01, 0.5, 0.5, 0.99]):
        _check_against_oracle(A, c, cal.astype(np.float64), test, alphas)
    out = torch.empty(len(cal), dtype=torch.float32, device="cuda")
    A.atts_calib_export(c, out)
    got = out.cpu().numpy()
    assert np.isnan(got[0]) and np.array_equal(got[1:], np.sort(cal[~np.isnan(cal)]))
    # empty test batch: only the thresholds are produced
    ranks, cls, p, q = _classify(A, c, np.zeros(0, np.float32), [0.3])
    assert len(ranks) == 0 and q[0] == O.quantile_thresholds(cal.astype(np.float64), O.reject_ranks([0.3], len(cal)))[0]


@pytest.mark.parametrize("sizes", [(1,), (7, 1, 300), (2047, 2048, 2049, 5), (8191, 8193, 5), (65536, 65537, 16, 65535),
                                   (20000, 3, 70001), (200000, 131072 + 17),
                                   # set sizes at and around whole index nodes (32, 1024, 32768 keys)
                                   (31, 1, 1, 991, 1, 31743, 1, 1)])
def test_online_appends_span_sort_chunks_and_merge_paths(sizes):
    """Batches below / at / above one sort run (8192 keys), the one-pass multi-way placement (up to 8 runs =
    65,536 keys) and the radix sort (larger batches, ragged last tile); after every append the state must equal
    the sorted union."""
    import paper_2509_15148_amd as A
    announce("calib appends", sizes)
    total = sum(sizes)
    allv = np.round(lognormal_scores(total, seed=sum(sizes)), 3)       # rounding plants many ties
    c = A.Calib(total)
    test = np.concatenate([lognormal_scores(500, seed=77), allv[:50]])
    lo = 0
    for s in sizes:
        A.atts_calibrate_online(c, dev(allv[lo:lo + s]))
        lo += s
        assert A.atts_calib_size(c) == lo
        out = torch.empty(lo, dtype=torch.float32, device="cuda")
        A.atts_calib_export(c, out)
        assert np.array_equal(out.cpu().numpy(), np.sort(allv[:lo]))
        _check_against_oracle(A, c, allv[:lo].astype(np.float64), test, [0.05, 0.2], brute=lo <= 30000)


def test_capacity_and_argument_errors():
    import paper_2509_15148_amd as A
    announce("calib errors")
    c = A.Calib(10)
    x = dev(np.arange(8, dtype=np.float32))
    with pytest.raises(A.AttsError) as e:                      # classify on an empty set
        _classify(A, c, np.zeros(3, np.float32), [0.1])
    assert e.value.code == A.ERR_INVALID_ARG
    A.atts_calibrate_online(c, x)
    with pytest.raises(A.AttsError) as e:
        A.atts_calibrate_online(c, x)
    assert e.value.code == A.ERR_CAPACITY and A.atts_calib_size(c) == 8
    A.atts_calibrate_online(c, x[:0])                          # empty append is a no-op
    for bad in ([], [0.0], [1.0], [0.3, 0.2], [0.1] * 9, [float("nan")]):
        with pytest.raises(A.AttsError) as e:
            _classify(A, c, np.zeros(3, np.float32), bad)
        assert e.value.code == A.ERR_INVALID_ARG
    with pytest.raises(A.AttsError) as e:                      # p-values need the ranks
        A.atts_classify_ordinal(c, x[:3], [0.5], None, torch.empty(3, device="cuda"), torch.empty(3, dtype=torch.uint8, device="cuda"), None)
    assert e.value.code == A.ERR_INVALID_ARG
    A.atts_calib_reset(c)
    assert A.atts_calib_size(c) == 0
    A.atts_calibrate_online(c, x[:3])
    _check_against_oracle(A, c, np.arange(3, dtype=np.float64), np.array([-1, 0, 1.5, 2, 9], np.float32), [0.5])


def test_calibration_only_workload_full_size():
    """The calibration-only workload at its published size: 2^20 lognormal scores, 16 online steps
    of 65,536 appended + 65,536 classified at alpha = (0.05, 0.2).  Every rank and class is checked
    against the oracle's sort-based count; 128 sampled test scores per step against the double sum."""
    import paper_2509_15148_amd as A
    wl = WORKLOADS["calib"]
    announce("calib full workload", wl.n_cal, wl.n_new, wl.n_steps)
    cal = lognormal_scores(wl.n_cal, wl.seed)
    c = A.Calib(wl.n_cal + wl.n_steps * wl.n_new)
    A.atts_calibrate_online(c, dev(cal))
    rng = np.random.default_rng(1)
    counts = np.zeros(3, dtype=np.int64)
    for step in range(wl.n_steps):
        new = lognormal_scores(wl.n_new, wl.seed + 1000 + step)
        test = lognormal_scores(wl.n_test, wl.seed + 2000 + step)
        A.atts_calibrate_online(c, dev(new))
        cal = np.concatenate([cal, new])
        ranks, cls, p, q = _classify(A, c, test, list(wl.alphas))
        cal64 = cal.astype(np.float64)
        cs = O.rank_counts_sorted(cal64, test)
        r = O.reject_ranks(wl.alphas, len(cal))
        assert np.array_equal(ranks.astype(np.int64), cs), step
        assert np.array_equal(cls, O.classify(cs, r)), step
        assert np.array_equal(q, O.quantile_thresholds(cal64, r).astype(np.float32))
        cls2 = torch.empty(wl.n_test, dtype=torch.uint8, device="cuda")
        A.atts_classify_ordinal(c, dev(test), list(wl.alphas), None, None, cls2, None)
        assert np.array_equal(cls2.cpu().numpy(), cls), step
        idx = rng.choice(wl.n_test, 128, replace=False)
        assert np.array_equal(ranks[idx].astype(np.int64), O.rank_counts(cal64, test[idx]))
        counts += np.bincount(cls, minlength=3)
    frac = counts / counts.sum()
    assert abs(frac[2] - 0.05) < 0.005 and abs(frac[1] + frac[2] - 0.2) < 0.01     # take-over rate ~ alpha


def test_streaming_merge_sizes():
    """Batches and totals above 2^22 keys take the streaming merge (4096-key segments, splits found by a
    separate kernel) in both its pairwise and its final form; smaller appends into the large set, ragged
    lengths and ties included.  The state must equal the sorted union after every append."""
    import paper_2509_15148_amd as A
    sizes = ((1 << 22) + 12345, 5_000_000, 70_001, 17, 8192)
    announce("calib streaming merge", sizes)
    total = sum(sizes)
    allv = np.round(lognormal_scores(total, seed=4242), 4)
    c = A.Calib(total)
    test = np.concatenate([lognormal_scores(4000, seed=78), allv[:96], np.array([0.0, np.inf, -1.0, np.nan], np.float32)])
    lo = 0
    for s in sizes:
        A.atts_calibrate_online(c, dev(allv[lo:lo + s]))
        lo += s
        out = torch.empty(lo, dtype=torch.float32, device="cuda")
        A.atts_calib_export(c, out)
        assert np.array_equal(out.cpu().numpy(), np.sort(allv[:lo])), s
        _check_against_oracle(A, c, allv[:lo].astype(np.float64), test, [0.05, 0.2], brute=False)
    idx = np.arange(0, len(test), 64)
    ranks = _classify(A, c, test[idx], [0.05, 0.2])[0]
    assert np.array_equal(ranks.astype(np.int64), O.rank_counts(allv.astype(np.float64), test[idx]))


@pytest.mark.parametrize("kind", ["lognormal", "clustered"])
def test_large_set_rank_search_with_guessed_window(kind):
    """Sets of 2^24 scores and more: the rank search first tries a two-line window picked by linear interpolation
    inside a 256-key block and falls back to the two index levels when the window does not bracket the score.
    Smooth data takes the window almost always; clustered data (long runs of equal scores, gaps of several orders of
    magnitude, sub-normals) defeats the guess.  Every rank and class against the oracle's sort-based count, sampled
    ones against the double sum."""
    import paper_2509_15148_amd as A
    n, m = (1 << 24) + 4321, 1 << 18
    announce("calib guessed window", kind, n, m)
    rng = np.random.default_rng(11)
    if kind == "lognormal":
        cal = lognormal_scores(n, seed=606)
        test = lognormal_scores(m, seed=607)
    else:
        parts = [np.full(n // 3, 1.0, np.float32), lognormal_scores(n // 3, seed=608) * np.float32(1e-30),
                 (rng.integers(0, 50, n - 2 * (n // 3)) * 1000.0).astype(np.float32)]
        cal = np.concatenate(parts)
        rng.shuffle(cal)
        test = np.concatenate([cal[: m // 2], lognormal_scores(m // 4, seed=609) * np.float32(1e-30),
                               (rng.random(m - m // 2 - m // 4) * 60000.0 - 5000.0).astype(np.float32)])
    c = A.Calib(n)
    A.atts_calibrate_online(c, dev(cal))
    ranks, cls, p, q = _classify(A, c, test, [0.05, 0.2])
    cal64 = cal.astype(np.float64)
    want = O.rank_counts_sorted(cal64, test)
    assert np.array_equal(ranks.astype(np.int64), want)
    r = O.reject_ranks([0.05, 0.2], n)
    assert np.array_equal(cls, O.classify(want, r))
    assert np.array_equal(q, O.quantile_thresholds(cal64, r).astype(np.float32))
    idx = rng.choice(m, 24, replace=False)
    assert np.array_equal(ranks[idx].astype(np.int64), O.rank_counts(cal64, test[idx]))


def test_out_of_cache_size_sampled():
    """2^28 resident scores + one append of 2^24 (the out-of-cache variant that bench.py times): the coarsest
    index level no longer fits LDS whole, so the strided top level + window search is exercised.  Ranks of
    sampled test scores against the oracle's double sum; the exported state must be ascending and keep every
    score (sum of ranks of the extreme probes)."""
    import paper_2509_15148_amd as A
    n0, n1 = 1 << 28, 1 << 24
    announce("calib out-of-cache", n0, n1)
    g = torch.Generator(device="cuda").manual_seed(99)
    cal0 = torch.randn(n0, device="cuda", generator=g).exp_()
    cal1 = torch.randn(n1, device="cuda", generator=g).exp_()
    c = A.Calib(n0 + n1)
    A.atts_calibrate_online(c, cal0)
    A.atts_calibrate_online(c, cal1)
    assert A.atts_calib_size(c) == n0 + n1
    out = torch.empty(n0 + n1, dtype=torch.float32, device="cuda")
    A.atts_calib_export(c, out)
    assert bool((out[1:] >= out[:-1]).all())
    del out
    host = np.concatenate([cal0.cpu().numpy(), cal1.cpu().numpy()])
    del cal0, cal1
    test = np.concatenate([lognormal_scores(60, seed=5), host[:3], np.array([0.0, 1e30], np.float32)]).astype(np.float32)
    ranks, cls, p, q = _classify(A, c, test, [0.05, 0.2])
    n = len(host)
    want = O.rank_counts(host.astype(np.float64), test)
    assert np.array_equal(ranks.astype(np.int64), want)
    r = O.reject_ranks([0.05, 0.2], n)
    assert np.array_equal(cls, O.classify(want, r))
    assert np.array_equal(p, O.p_values(want, n).astype(np.float32))
    assert ranks[-2] == n and ranks[-1] == 0
    # thresholds: the (n + 1 - r)-th smallest, by partition instead of a full sort
    for l in range(2):
        kth = n + 1 - int(r[l])
        assert q[l] == np.partition(host, kth - 1)[kth - 1]


def test_export_import_round_trip():
    """Checkpoint / resume of the online calibration state: a handle restored from an export gives the same ranks,
    classes and thresholds bit for bit, before and after further appends to both."""
    import paper_2509_15148_amd as A
    announce("calib export/import")
    for n0, n1 in ((16, 5), (1000, 37), (70000, 9000), (300000, 70001)):
        cal = lognormal_scores(n0, 901).astype(np.float32)
        cal[:: max(n0 // 7, 1)] = cal[0]
        if n0 > 100:
            cal[3], cal[5], cal[9], cal[11] = np.nan, -0.0, 0.0, np.inf
        more = lognormal_scores(n1, 902).astype(np.float32)
        test = np.concatenate([lognormal_scores(3000, 903).astype(np.float32), cal[:50],
                               np.array([np.nan, 0.0, -0.0, np.inf, -np.inf], dtype=np.float32)])
        alphas = [0.05, 0.2]
        a = A.Calib(n0 + n1)
        A.atts_calibrate_online(a, dev(cal[: n0 // 2]))
        A.atts_calibrate_online(a, dev(cal[n0 // 2:]))
        saved = torch.empty(n0, dtype=torch.float32, device="cuda")
        A.atts_calib_export(a, saved)
        b = A.Calib(n0 + n1)
        A.atts_calibrate_online(b, dev(more))                     # old contents are replaced by the import
        A.atts_calib_import(b, saved)
        assert A.atts_calib_size(b) == n0
        ra = _classify(A, a, test, alphas)
        rb = _classify(A, b, test, alphas)
        for x, y in zip(ra, rb):
            assert np.array_equal(x, y, equal_nan=True)
        _check_against_oracle(A, b, cal.astype(np.float64), test, alphas, brute=n0 <= 1000)
        A.atts_calibrate_online(a, dev(more))
        A.atts_calibrate_online(b, dev(more))
        ra = _classify(A, a, test, alphas)
        rb = _classify(A, b, test, alphas)
        for x, y in zip(ra, rb):
            assert np.array_equal(x, y, equal_nan=True)
        with pytest.raises(A.AttsError) as e:
            A.atts_calib_import(b, torch.zeros(n0 + n1 + 1, dtype=torch.float32, device="cuda"))
        assert e.value.code == A.ERR_CAPACITY
        A.atts_calib_import(b, torch.zeros(0, dtype=torch.float32, device="cuda"))
        assert A.atts_calib_size(b) == 0
        a.close()
        b.close()
