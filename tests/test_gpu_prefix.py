"""The prefix handle: scoring against cached prefix keys / values must give what scoring the whole token tree
gives (and what the oracle gives), whatever the split into prefill / extend calls."""
import numpy as np
import pytest
import torch

from oracle import atts_oracle as O
from synth import WORKLOADS, ModelConfig, make_token_ids, make_weights
from util import announce, dev, weights_to_numpy, ws

pytestmark = pytest.mark.gpu

TOL = {"fp32": 1e-4, "bf16": 2e-2}


def _cold(A, model, prefix, drafts, lens=None):
    K, T = drafts.shape
    lp = torch.full((K, T), float("nan"), dtype=torch.float32, device="cuda")
    sc = torch.full((K,), float("nan"), dtype=torch.float32, device="cuda")
    A.atts_score_drafts(model, dev(prefix), dev(drafts), None if lens is None else dev(lens), 0, lp, sc,
                        ws(A.atts_workspace_bytes(model, len(prefix), K, T)))
    torch.cuda.synchronize()
    return lp.cpu().numpy(), sc.cpu().numpy()


def _cached(A, model, pre, drafts, lens=None, mode=0):
    K, T = drafts.shape
    lp = torch.full((K, T), float("nan"), dtype=torch.float32, device="cuda")
    sc = torch.full((K,), float("nan"), dtype=torch.float32, device="cuda")
    A.atts_score_drafts_cached(pre, dev(drafts), None if lens is None else dev(lens), mode, lp, sc,
                               ws(A.atts_workspace_bytes(model, A.atts_prefix_length(pre), K, T)))
    torch.cuda.synchronize()
    return lp.cpu().numpy(), sc.cpu().numpy()


def _extend(A, pre, ids):
    A.atts_prefix_extend(pre, dev(ids), ws(A.atts_prefix_extend_workspace_bytes(pre, len(ids))))


@pytest.mark.parametrize("cfg,P,K,T,chunks", [
    (WORKLOADS["tiny"].model, 64, 8, 32, (64,)),                                   # fp32, simple attention
    (ModelConfig(2, 96, 4, 1, 24, 200, 515, "fp32"), 19, 4, 23, (7, 1, 11)),        # prefill in three pieces
    (ModelConfig(2, 256, 4, 2, 128, 520, 2003, "bf16"), 70, 3, 45, (70,)),          # MFMA attention, general GEMM
    (ModelConfig(2, 256, 4, 2, 128, 512, 2048, "bf16"), 72, 5, 40, (40, 32)),       # aligned GEMM + fused RoPE epilogue
    (ModelConfig(2, 256, 4, 2, 128, 512, 2048, "bf16"), 130, 2, 9, (1, 129)),       # prefix length not a multiple of 4
])
def test_cached_scoring_matches_cold_scoring_and_the_oracle(cfg, P, K, T, chunks):
    import paper_2509_15148_amd as A
    announce("prefix handle", cfg, P, K, T, chunks)
    w_dev = make_weights(cfg, seed=P * 31 + K, device="cuda")
    prefix, drafts = make_token_ids(cfg.vocab, P, K, T, P + 7 * K)
    prefix, drafts = prefix.numpy(), drafts.numpy()
    model = A.Model(cfg, w_dev)
    pre = A.Prefix(model, capacity=P + 5)
    lo = 0
    for n in chunks:
        _extend(A, pre, prefix[lo:lo + n])
        lo += n
    assert lo == P and A.atts_prefix_length(pre) == P
    lens = np.array([max(1, T - 3 * k) for k in range(K)], dtype=np.int32)
    for ln in (None, lens):
        lp_c, sc_c = _cold(A, model, prefix, drafts, ln)
        lp_w, sc_w = _cached(A, model, pre, drafts, ln)
        ref_lp, ref_s = O.score_drafts(weights_to_numpy(w_dev), cfg, prefix, drafts, draft_lens=ln)
        tol = TOL[cfg.dtype]
        assert np.abs(lp_w - ref_lp).max() <= tol and np.abs(sc_w - ref_s).max() <= tol
        # cached and cold differ only by where the query tiles of the attention kernel start (bf16 rounding of
        # the probabilities is then grouped differently): well inside the tolerance
        assert np.abs(lp_w - lp_c).max() <= tol / 2, np.abs(lp_w - lp_c).max()
    # a second call on the same handle gives the same result, bit for bit (the handle is not modified by scoring; the
    # partial sums of projections that split their K range are added in a fixed order)
    lp_w2, _ = _cached(A, model, pre, drafts, lens)
    assert np.array_equal(lp_w, lp_w2)
    assert A.atts_model_check(model) == 0


def test_extend_with_an_accepted_draft_then_score_the_next_turn():
    """Turn t + 1: the accepted continuation joins the prefix; new drafts are scored against prefix + continuation."""
    import paper_2509_15148_amd as A
    cfg = ModelConfig(2, 256, 4, 2, 128, 512, 2048, "bf16")
    announce("prefix extend turn", cfg)
    w_dev = make_weights(cfg, seed=77, device="cuda")
    prefix, drafts1 = [x.numpy() for x in make_token_ids(cfg.vocab, 48, 4, 20, 1)]
    _, drafts2 = [x.numpy() for x in make_token_ids(cfg.vocab, 48, 3, 17, 2)]
    model = A.Model(cfg, w_dev)
    pre = A.Prefix(model, capacity=48 + 20)
    _extend(A, pre, prefix)
    _cached(A, model, pre, drafts1)
    _extend(A, pre, drafts1[2])                                   # draft 2 of turn 1 is accepted
    assert A.atts_prefix_length(pre) == 68
    lp_w, sc_w = _cached(A, model, pre, drafts2)
    ctx = np.concatenate([prefix, drafts1[2]])
    ref_lp, ref_s = O.score_drafts(weights_to_numpy(w_dev), cfg, ctx, drafts2)
    assert np.abs(lp_w - ref_lp).max() <= TOL["bf16"] and np.abs(sc_w - ref_s).max() <= TOL["bf16"]
    with pytest.raises(A.AttsError) as e:                         # the handle is full
        _extend(A, pre, prefix[:1])
    assert e.value.code == A.ERR_CAPACITY and A.atts_prefix_length(pre) == 68
    A.atts_prefix_reset(pre)
    assert A.atts_prefix_length(pre) == 0
    with pytest.raises(A.AttsError) as e:                         # nothing to score against
        _cached(A, model, pre, drafts2)
    assert e.value.code == A.ERR_INVALID_ARG


def test_7b_width_cached_prefix_sampled_draft():
    """The 7B-class workload with its 512-token prefix cached (two layers): all K drafts on the GPU, one sampled
    draft through the oracle as a plain causal sequence."""
    import paper_2509_15148_amd as A
    wl = WORKLOADS["7b"]
    cfg = wl.model
    announce("prefix handle 7b width")
    w_dev = make_weights(cfg, wl.seed, device="cuda", n_layers=2)
    prefix, drafts = [x.numpy() for x in make_token_ids(cfg.vocab, wl.P, wl.K, wl.T, wl.seed)]
    model = A.Model(cfg, w_dev)
    pre = A.Prefix(model, capacity=wl.P)
    _extend(A, pre, prefix)
    lp_w, sc_w = _cached(A, model, pre, drafts)
    lp_c, sc_c = _cold(A, model, prefix, drafts)
    assert np.abs(lp_w - lp_c).max() <= 1e-2
    w_np = weights_to_numpy(w_dev)
    ref = O.token_logprobs(w_np, cfg, prefix, drafts[9])
    assert np.abs(lp_w[9] - ref).max() <= TOL["bf16"]
    assert abs(sc_w[9] - O.conformity_score(ref)) <= TOL["bf16"]
