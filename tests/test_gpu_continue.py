"""Greedy target-model continuation ("Target Model Sampling") against the oracle's arg-max chain.

The token decided at a step is an arg max over floating-point logits: where the oracle's best and second-best
logits are closer than the accuracy of the GPU arithmetic, either token is a correct decision; the comparison
therefore requires equal tokens wherever the oracle's margin exceeds a tolerance, and after a (permitted)
divergence the rest of that candidate is not compared (its context differs)."""
import numpy as np
import pytest
import torch

from oracle import atts_oracle as O
from synth import WORKLOADS, ModelConfig, make_token_ids, make_weights
from util import announce, dev, weights_to_numpy, ws

pytestmark = pytest.mark.gpu

MARGIN = {"fp32": 1e-3, "bf16": 0.15}      # logits here are O(1): bf16 rounding through the model moves them by a few 1e-2


def _continue(A, model, prefix, drafts, n_new, chunks=None):
    pre = A.Prefix(model, capacity=len(prefix))
    lo = 0
    for n in (chunks or (len(prefix),)):
        A.atts_prefix_extend(pre, dev(prefix[lo:lo + n]), ws(A.atts_prefix_extend_workspace_bytes(pre, n)))
        lo += n
    K, T = drafts.shape
    out = torch.full((K, n_new), -1, dtype=torch.int32, device="cuda")
    A.atts_continue_greedy(pre, dev(drafts), out, ws(A.atts_continue_workspace_bytes(pre, K, T, n_new)))
    torch.cuda.synchronize()
    return out.cpu().numpy(), pre


def _compare(cfg, w_np, prefix, drafts, got, n_new):
    agree = 0
    for k in range(drafts.shape[0]):
        ref, margins = O.greedy_continuation(w_np, cfg, prefix, drafts[k], n_new)
        for t in range(n_new):
            if got[k, t] == ref[t]:
                agree += 1
                continue
            assert margins[t] <= MARGIN[cfg.dtype], (k, t, int(got[k, t]), int(ref[t]), margins[t])
            # the GPU's token must itself be a near-maximum of the oracle's distribution at that step
            ctx = np.concatenate([prefix, drafts[k], ref[:t]])
            lp = O.token_logprobs(w_np, cfg, ctx, np.array([got[k, t], ref[t]]))
            # (second entry is conditioned on the first; only the first matters here)
            best = O.token_logprobs(w_np, cfg, ctx, ref[t:t + 1])[0]
            assert best - lp[0] <= MARGIN[cfg.dtype]
            break
    return agree


@pytest.mark.parametrize("cfg,P,K,T,n_new,chunks", [
    (WORKLOADS["tiny"].model, 24, 3, 9, 6, None),                                   # fp32, simple attention
    (ModelConfig(2, 96, 4, 1, 24, 200, 515, "fp32"), 7, 2, 5, 8, (3, 4)),
    (ModelConfig(2, 256, 4, 2, 128, 512, 2048, "bf16"), 40, 4, 12, 6, None),         # bf16, transposed-value prefix cache
    (ModelConfig(2, 256, 4, 2, 128, 520, 2003, "bf16"), 33, 2, 7, 5, (32, 1)),       # general GEMM path
    # decode attention by 16-byte pieces: 8 / 32 / 8 lanes per key, and contexts beyond the batches requested up front
    (ModelConfig(2, 128, 4, 2, 32, 192, 515, "fp32"), 70, 3, 20, 4, None),
    (ModelConfig(2, 256, 2, 1, 128, 256, 515, "fp32"), 500, 2, 6, 4, None),
    (ModelConfig(2, 256, 4, 2, 64, 512, 2048, "bf16"), 300, 3, 10, 4, None),
    (ModelConfig(2, 256, 4, 2, 128, 512, 2048, "bf16"), 950, 2, 8, 4, None),
    # more candidates than the 16-row kernel takes: the decoding steps go through the tiled GEMMs
    (ModelConfig(2, 256, 4, 2, 128, 512, 2048, "bf16"), 20, 20, 4, 3, None),
    (ModelConfig(2, 96, 4, 1, 24, 200, 515, "fp32"), 6, 18, 3, 3, None),
])
def test_greedy_continuation_matches_the_oracle(cfg, P, K, T, n_new, chunks):
    import paper_2509_15148_amd as A
    announce("continue greedy", cfg, P, K, T, n_new)
    w_dev = make_weights(cfg, seed=P * 13 + K, device="cuda")
    prefix, drafts = [x.numpy() for x in make_token_ids(cfg.vocab, P, K, T, P + K)]
    model = A.Model(cfg, w_dev)
    got, pre = _continue(A, model, prefix, drafts, n_new, chunks)
    assert got.min() >= 0 and got.max() < cfg.vocab
    agree = _compare(cfg, weights_to_numpy(w_dev), prefix, drafts, got, n_new)
    assert agree >= K * n_new // 2                       # most decisions are clear-cut and must agree exactly
    assert A.atts_prefix_length(pre) == P and A.atts_model_check(model) == 0
    # n_new = 1 is the first token of the longer run, and a second full run reproduces the first token for token (every
    # sum is taken in a fixed order)
    got1, _ = _continue(A, model, prefix, drafts, 1, chunks)
    assert np.array_equal(got1[:, 0], got[:, 0])
    got2, _ = _continue(A, model, prefix, drafts, n_new, chunks)
    assert np.array_equal(got2, got)


SLACK = {"fp32": 2e-4, "bf16": 0.05}        # how close (in probability) a draw may be to a CDF boundary for the tokens to differ


def _check_sampled(cfg, w_np, prefix, draft, u_row, temperature, got_row, tol, eos_id=None):
    """One candidate's sampled tokens against the oracle's chain for the same draws.  Returns the number of leading
    tokens that agree.  At the first token that differs, the GPU's token must be one the draw could have picked
    within the arithmetic's accuracy: the interval (cdf[v - 1], cdf[v]] that the ORACLE's distribution gives the
    GPU's token v must lie within `tol` (in probability) of the draw; the rest of the candidate is then not
    compared (its context differs)."""
    ref, _ = O.sampled_continuation(w_np, cfg, prefix, draft, np.asarray(u_row, dtype=np.float64), temperature, eos_id=eos_id)
    for t in range(len(ref)):
        if int(got_row[t]) == int(ref[t]):
            continue
        cdf = O.next_token_cdf(w_np, cfg, np.concatenate([prefix, draft, ref[:t]]), temperature)
        v, u = int(got_row[t]), float(u_row[t])
        lo, hi = (cdf[v - 1] if v > 0 else 0.0), cdf[v]
        dist = max(lo - u, u - hi, 0.0)
        assert dist <= tol, (t, v, int(ref[t]), u, lo, hi, dist)
        return t
    return len(ref)


def _guided_uniforms(cfg, w_np, prefix, draft, n_new, temperature, rng):
    """Draws for one candidate chosen with the oracle so that most of them are clear decisions: at every step the
    draw is the midpoint of the CDF interval of one of the oracle's most probable tokens (picked at random among
    those that hold at least a fifth of the largest mass), rounded to fp32; the chain then follows the oracle's
    own choice for that draw.  Every other step keeps a plain uniform draw instead."""
    us, ctx = [], np.concatenate([prefix, draft])
    for t in range(n_new):
        cdf = O.next_token_cdf(w_np, cfg, ctx, temperature)
        mass = np.diff(np.concatenate([[0.0], cdf]))
        if t % 2 == 0:
            big = np.flatnonzero(mass >= 0.2 * mass.max())
            v = int(big[rng.integers(len(big))])
            u = np.float32((cdf[v] - 0.5 * mass[v]))
        else:
            u = np.float32(rng.random())
        u = float(min(u, np.float32(1.0 - 2.0 ** -24)))
        v = min(int(np.searchsorted(cdf, u, side="left")), len(cdf) - 1)
        us.append(u)
        ctx = np.concatenate([ctx, [v]])
    return np.asarray(us, dtype=np.float32)


@pytest.mark.parametrize("cfg,P,K,T,n_new,temperature", [
    (WORKLOADS["tiny"].model, 24, 3, 9, 6, 1.0),
    (ModelConfig(2, 96, 4, 1, 24, 200, 515, "fp32"), 7, 4, 5, 5, 0.7),
    (ModelConfig(2, 256, 4, 2, 128, 512, 2048, "bf16"), 40, 4, 12, 5, 1.3),
])
def test_sampled_continuation_matches_the_oracle(cfg, P, K, T, n_new, temperature):
    """Inverse-CDF sampling with the same uniforms on both sides; a token may differ only where the draw lies within
    the arithmetic's accuracy of a boundary between two tokens' CDF intervals (then the rest of that candidate is
    not compared)."""
    import paper_2509_15148_amd as A
    announce("continue sample", cfg, P, K, T, n_new, temperature)
    w_dev = make_weights(cfg, seed=P * 17 + K, device="cuda")
    prefix, drafts = [x.numpy() for x in make_token_ids(cfg.vocab, P, K, T, P + 3 * K)]
    model = A.Model(cfg, w_dev)
    pre = A.Prefix(model, capacity=P)
    A.atts_prefix_extend(pre, dev(prefix), ws(A.atts_prefix_extend_workspace_bytes(pre, P)))
    rng = np.random.default_rng(P + K)
    u = rng.random((K, n_new)).astype(np.float32)
    u[0, 0] = 0.0
    out = torch.full((K, n_new), -1, dtype=torch.int32, device="cuda")
    A.atts_continue_sample(pre, dev(drafts), temperature, dev(u), out, ws(A.atts_continue_workspace_bytes(pre, K, T, n_new)))
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert got.min() >= 0 and got.max() < cfg.vocab
    w_np = weights_to_numpy(w_dev)
    agree = sum(_check_sampled(cfg, w_np, prefix, drafts[k], u[k], temperature, got[k], SLACK[cfg.dtype]) for k in range(K))
    assert agree >= K * n_new // 2
    # different uniforms give different continuations (the draws are really used)
    out2 = torch.empty_like(out)
    A.atts_continue_sample(pre, dev(drafts), temperature, dev(1.0 - 1e-3 - u * 0.5), out2, ws(A.atts_continue_workspace_bytes(pre, K, T, n_new)))
    assert not torch.equal(out, out2)
    for bad_t in (0.0, -1.0, float("inf"), float("nan")):
        with pytest.raises(A.AttsError) as e:
            A.atts_continue_sample(pre, dev(drafts), bad_t, dev(u), out, ws(A.atts_continue_workspace_bytes(pre, K, T, n_new)))
        assert e.value.code == A.ERR_INVALID_ARG


def test_7b_width_continuation():
    """Full 7B width (two layers): the aligned few-row GEMM path (128-row tiles, K-split projections), the
    transposed-value prefix cache and a vocabulary of 152,064 in the arg max."""
    import paper_2509_15148_amd as A
    wl = WORKLOADS["7b"]
    cfg = wl.model
    P, K, T, n_new = 24, 2, 6, 3
    announce("continue greedy 7b width", P, K, T, n_new)
    w_dev = make_weights(cfg, wl.seed, device="cuda", n_layers=2)
    prefix, drafts = [x.numpy() for x in make_token_ids(cfg.vocab, P, K, T, 99)]
    model = A.Model(cfg, w_dev)
    got, _ = _continue(A, model, prefix, drafts, n_new)
    assert got.min() >= 0 and got.max() < cfg.vocab
    w_np = weights_to_numpy(w_dev)
    agree = _compare(cfg, w_np, prefix, drafts, got, n_new)
    assert agree >= K * n_new // 2
    # sampling over the same vocabulary.  With 152,064 tokens of O(1) logits a plain draw at temperature 1 lands in
    # an interval 1e-5 wide, which no bf16 model can resolve; at temperature 0.1 the few most probable tokens hold most of
    # the mass, and the draws are chosen with the oracle (midpoints of wide intervals, alternating with plain
    # uniforms) so that most decisions are clear.  A token that differs must still be one the draw could have
    # picked within the bf16 accuracy.
    pre = A.Prefix(model, capacity=P)
    A.atts_prefix_extend(pre, dev(prefix), ws(A.atts_prefix_extend_workspace_bytes(pre, P)))
    temperature = 0.1
    rng = np.random.default_rng(7)
    u = np.stack([_guided_uniforms(cfg, w_np, prefix, drafts[k], n_new, temperature, rng) for k in range(K)])
    out = torch.full((K, n_new), -1, dtype=torch.int32, device="cuda")
    A.atts_continue_sample(pre, dev(drafts), temperature, dev(u), out, ws(A.atts_continue_workspace_bytes(pre, K, T, n_new)))
    torch.cuda.synchronize()
    got_s = out.cpu().numpy()
    assert got_s.min() >= 0 and got_s.max() < cfg.vocab
    agree_s = sum(_check_sampled(cfg, w_np, prefix, drafts[k], u[k], temperature, got_s[k], SLACK["bf16"]) for k in range(K))
    assert agree_s >= K * n_new // 2, (agree_s, got_s)


@pytest.mark.timeout(900)
def test_7b_width_continuation_at_the_benchmark_shape():
    """The continuation leg bench.py times: 7B width (two layers), a 512-token prefix cached, 4 rejected candidates
    with 256-token drafts, 4 new tokens each (context pass over 1024 draft rows, then three decoding steps of 4
    rows).  The oracle runs every candidate as its own plain causal sequence."""
    import paper_2509_15148_amd as A
    wl = WORKLOADS["7b"]
    cfg = wl.model
    P, K, T, n_new = wl.P, 4, wl.T, 4
    announce("continue greedy 7b width, benchmark shape", P, K, T, n_new)
    w_dev = make_weights(cfg, wl.seed, device="cuda", n_layers=2)
    prefix, drafts = [x.numpy() for x in make_token_ids(cfg.vocab, P, K, T, wl.seed + 700001)]
    model = A.Model(cfg, w_dev)
    got, _ = _continue(A, model, prefix, drafts, n_new)
    assert got.min() >= 0 and got.max() < cfg.vocab and A.atts_model_check(model) == 0
    w_np = weights_to_numpy(w_dev)
    del w_dev, model
    torch.cuda.empty_cache()
    agree = _compare(cfg, w_np, prefix, drafts, got, n_new)
    print(f"[continue 7b bench shape] {agree} of {K * n_new} decisions equal", flush=True)
    assert agree >= K * n_new // 2


def test_continuation_argument_errors():
    import paper_2509_15148_amd as A
    cfg = WORKLOADS["tiny"].model
    announce("continue errors")
    w_dev = make_weights(cfg, seed=5, device="cuda")
    model = A.Model(cfg, w_dev)
    pre = A.Prefix(model, capacity=8)
    drafts = dev(np.zeros((2, 3), np.int32))
    out = torch.zeros((2, 4), dtype=torch.int32, device="cuda")
    with pytest.raises(A.AttsError) as e:                          # empty prefix
        A.atts_continue_workspace_bytes(pre, 2, 3, 4)
    assert e.value.code == A.ERR_INVALID_ARG
    A.atts_prefix_extend(pre, dev(np.arange(5, dtype=np.int32)), ws(A.atts_prefix_extend_workspace_bytes(pre, 5)))
    need = A.atts_continue_workspace_bytes(pre, 2, 3, 4)
    with pytest.raises(A.AttsError) as e:
        A.atts_continue_greedy(pre, drafts, out, ws(need - 256))
    assert e.value.code == A.ERR_WORKSPACE
    for K, T, n in ((0, 3, 4), (2, 0, 4), (2, 3, 0), (769, 3, 4)):
        with pytest.raises(A.AttsError) as e:
            A.atts_continue_workspace_bytes(pre, K, T, n)
        assert e.value.code == A.ERR_INVALID_ARG


@pytest.mark.parametrize("cfg,P,T,lens,n_new", [
    (ModelConfig(2, 96, 4, 1, 24, 200, 515, "fp32"), 9, 7, (7, 1, 4), 6),                 # general attention kernel
    (ModelConfig(2, 256, 4, 2, 128, 512, 2048, "bf16"), 40, 12, (3, 12, 8, 1), 6),       # pieces kernel, few-row GEMM
    (ModelConfig(2, 256, 2, 1, 128, 256, 515, "fp32"), 450, 30, (30, 2), 4),             # branches on both sides of a key batch
])
def test_ragged_drafts_and_end_of_sequence(cfg, P, T, lens, n_new):
    """Candidates of different lengths continue after their own last token (the padding of their rows, here out-of-
    vocabulary garbage, is never read), and a candidate that has produced the end token stays ended."""
    import paper_2509_15148_amd as A
    K = len(lens)
    announce("continue ragged", cfg, P, K, T, lens, n_new)
    w_dev = make_weights(cfg, seed=P + 5 * K, device="cuda")
    w_np = weights_to_numpy(w_dev)
    prefix, drafts = [x.numpy() for x in make_token_ids(cfg.vocab, P, K, T, 7 * P + K)]
    padded = drafts.copy()
    for k, n in enumerate(lens):
        padded[k, n:] = cfg.vocab + 17                      # must never be embedded
    model = A.Model(cfg, w_dev)
    pre = A.Prefix(model, capacity=P)
    A.atts_prefix_extend(pre, dev(prefix), ws(A.atts_prefix_extend_workspace_bytes(pre, P)))
    lens_dev = dev(np.asarray(lens, dtype=np.int32))
    out = torch.full((K, n_new), -1, dtype=torch.int32, device="cuda")
    wsb = A.atts_continue_workspace_bytes(pre, K, T, n_new)
    A.atts_continue_greedy(pre, dev(padded), out, ws(wsb), draft_lens=lens_dev)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert A.atts_model_check(model) == 0
    agree = 0
    for k, n in enumerate(lens):
        ref, margins = O.greedy_continuation(w_np, cfg, prefix, drafts[k, :n], n_new)
        for t in range(n_new):
            if got[k, t] != ref[t]:
                assert margins[t] <= MARGIN[cfg.dtype], (k, t, int(got[k, t]), int(ref[t]), margins[t])
                break
            agree += 1
    assert agree >= K * n_new // 2
    # end of sequence: take the token candidate 0 produced at step 1 as the end token
    eos = int(got[0, 1])
    out_e = torch.full((K, n_new), -1, dtype=torch.int32, device="cuda")
    A.atts_continue_greedy(pre, dev(padded), out_e, ws(wsb), draft_lens=lens_dev, eos_id=eos)
    torch.cuda.synchronize()
    got_e = out_e.cpu().numpy()
    for k in range(K):
        hits = np.flatnonzero(got[k] == eos)
        if len(hits) == 0:
            if not np.array_equal(got_e[k], got[k]):        # only a near-tie may move a token between two runs
                t = int(np.flatnonzero(got_e[k] != got[k])[0])
                _, m = O.greedy_continuation(w_np, cfg, prefix, np.concatenate([drafts[k, :lens[k]], got[k, :t]]), 1)
                assert m[0] <= MARGIN[cfg.dtype]
            continue
        first = int(hits[0])
        if np.array_equal(got_e[k, :first + 1], got[k, :first + 1]):
            assert np.all(got_e[k, first + 1:] == eos), (k, got_e[k], got[k])
    assert np.all(got_e[0, 2:] == eos) or got_e[0, 1] != eos
    # sampled: the same freezing rule, uniforms of the frozen positions unused
    u = np.random.default_rng(K).random((K, n_new)).astype(np.float32)
    out_s = torch.full((K, n_new), -1, dtype=torch.int32, device="cuda")
    A.atts_continue_sample(pre, dev(padded), 1.0, dev(u), out_s, ws(wsb), draft_lens=lens_dev)
    torch.cuda.synchronize()
    got_s = out_s.cpu().numpy()
    eos_s = int(got_s[K - 1, 0])
    A.atts_continue_sample(pre, dev(padded), 1.0, dev(u), out_s, ws(wsb), draft_lens=lens_dev, eos_id=eos_s)
    torch.cuda.synchronize()
    got_se = out_s.cpu().numpy()
    if got_se[K - 1, 0] == eos_s:
        assert np.all(got_se[K - 1] == eos_s)
    for k, n in enumerate(lens):
        _check_sampled(cfg, w_np, prefix, drafts[k, :n], u[k], 1.0, got_se[k], SLACK[cfg.dtype], eos_id=eos_s)
