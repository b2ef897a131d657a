"""Pins for the oracle's target-model forward pass and log-prob extraction.

The paper prints no numeric example for the verification forward pass, so it is pinned to
closed forms of degenerate models, to structural invariants of a causal decoder, and to
an independent float64 formulation assembled from torch library routines (rms_norm,
scaled_dot_product_attention with grouped KV heads, silu, log_softmax) with the rotary
embedding written as a complex multiplication.
"""
import copy
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import atts_oracle as O
from synth import ModelConfig, make_token_ids, make_weights
from util import weights_to_numpy

CFG = ModelConfig(n_layers=2, d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8, d_ffn=48,
                  vocab=50, dtype="fp32")


def _weights(cfg=CFG, seed=5, **kw):
    w = make_weights(cfg, seed, **kw)
    return {k: ([t.numpy() for t in v] if isinstance(v, list) else v.numpy()) for k, v in w.items()}


def _ids(cfg=CFG, P=9, K=3, T=6, seed=77):
    p, d = make_token_ids(cfg.vocab, P, K, T, seed)
    return p.numpy(), d.numpy()


# ---------------------------------------------------------------- log-softmax closed forms
def test_log_softmax_rows_sum_to_one_and_shift_invariance():
    z = np.random.default_rng(0).normal(scale=30.0, size=(7, 1000))
    lsm = O.log_softmax(z)
    assert np.allclose(np.exp(lsm).sum(-1), 1.0, rtol=0, atol=1e-12)
    assert np.all(lsm <= 0)
    assert np.allclose(O.log_softmax(z + 1e3), lsm, rtol=0, atol=1e-9)
    assert np.allclose(lsm, torch.log_softmax(torch.from_numpy(z), -1).numpy(), rtol=0, atol=1e-12)


def test_zero_lm_head_gives_uniform_distribution():
    w = _weights()
    w["lm_head"] = np.zeros_like(w["lm_head"])
    p, d = _ids()
    lp = O.token_logprobs(w, CFG, p, d[0])
    assert np.allclose(lp, -math.log(CFG.vocab), rtol=0, atol=1e-14)
    lps, s = O.score_drafts(w, CFG, p, d)
    assert np.allclose(s, math.log(CFG.vocab))            # mean NLL of a uniform model


# ---------------------------------------------------------------- degenerate models
def test_zero_output_projections_make_layers_identity():
    w = _weights()
    w["wo"] = [np.zeros_like(x) for x in w["wo"]]
    w["w_down"] = [np.zeros_like(x) for x in w["w_down"]]
    p, d = _ids()
    seq = np.concatenate([p, d[1]])
    h = O.decoder_hidden(w, CFG, seq)
    assert np.array_equal(h, w["tok_embed"][seq].astype(np.float64))
    x = torch.from_numpy(h)
    z = F.rms_norm(x, (CFG.d_model,), torch.from_numpy(w["final_norm"]).double(), CFG.rms_eps) \
        @ torch.from_numpy(w["lm_head"]).double().T
    ref = torch.log_softmax(z, -1).numpy()
    lp = O.token_logprobs(w, CFG, p, d[1])
    P = len(p)
    assert np.allclose(lp, ref[np.arange(P - 1, P - 1 + len(d[1])), d[1]], rtol=0, atol=1e-12)


def test_zero_layers_model():
    cfg = ModelConfig(0, 32, 4, 2, 8, 48, 50, "fp32")
    w = _weights(cfg)
    assert len(w["wqkv"]) == 0
    p, d = _ids(cfg)
    seq = np.concatenate([p, d[0]])
    assert np.array_equal(O.decoder_hidden(w, cfg, seq), w["tok_embed"][seq].astype(np.float64))


def test_uniform_attention_closed_form_and_gqa_head_mapping():
    """Zero query projection => every softmax is uniform over the causal window, so the
    context of query head j at position i is the running mean of V of KV head j // group."""
    cfg = ModelConfig(1, 32, 4, 2, 8, 48, 50, "fp32")
    w = _weights(cfg)
    nq, nkv, hd = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    w["wqkv"][0][: nq * hd] = 0.0
    w["w_down"][0][:] = 0.0
    p, d = _ids(cfg)
    seq = np.concatenate([p, d[0]])
    n = len(seq)
    e = torch.from_numpy(w["tok_embed"][seq]).double()
    a = F.rms_norm(e, (cfg.d_model,), torch.from_numpy(w["attn_norm"][0]).double(), cfg.rms_eps)
    v = (a @ torch.from_numpy(w["wqkv"][0][(nq + nkv) * hd:]).double().T).view(n, nkv, hd)
    run_mean = torch.cumsum(v, 0) / torch.arange(1, n + 1).double()[:, None, None]
    ctx = torch.stack([run_mean[:, j // (nq // nkv)] for j in range(nq)], 1).reshape(n, nq * hd)
    expect = e + ctx @ torch.from_numpy(w["wo"][0]).double().T
    got = O.decoder_hidden(w, cfg, seq)
    assert np.allclose(got, expect.numpy(), rtol=0, atol=1e-12)


# ---------------------------------------------------------------- structural invariants
def test_causality_and_prefix_split_invariance():
    w = _weights()
    p, d = _ids(P=9, T=6)
    lp = O.token_logprobs(w, CFG, p, d[0])
    d2 = d[0].copy()
    d2[-1] = (d2[-1] + 1) % CFG.vocab
    lp2 = O.token_logprobs(w, CFG, p, d2)
    assert np.allclose(lp[:-1], lp2[:-1], rtol=0, atol=1e-13)      # later tokens cannot leak back
    assert abs(lp[-1] - lp2[-1]) > 1e-6
    # moving the split point: (P, T) vs (P - j, j + T) agree on the common tokens
    for j in (1, 4):
        lp_shift = O.token_logprobs(w, CFG, p[:-j], np.concatenate([p[-j:], d[0]]))
        assert np.allclose(lp_shift[j:], lp, rtol=0, atol=1e-12)


def test_shared_prefix_tree_equals_independent_sequences():
    """Scoring K drafts under one prefix == K independent causal sequences; in particular
    the first draft token is predicted from the last prefix position, shared by all."""
    w = _weights()
    p, d = _ids(K=3)
    lps, s = O.score_drafts(w, CFG, p, d)
    h_prefix = O.decoder_hidden(w, CFG, p)
    first = O.log_softmax(O.logits_from_hidden(w, CFG, h_prefix[-1:]))[0]
    for k in range(3):
        assert np.allclose(lps[k, 0], first[d[k, 0]], rtol=0, atol=1e-12)
    lps_r, s_r = O.score_drafts(w, CFG, p, d[::-1])
    assert np.allclose(s_r[::-1], s, rtol=0, atol=1e-13)
    assert np.allclose(s, -lps.mean(1))
    _, s_sum = O.score_drafts(w, CFG, p, d, mode=O.SUM_NLL)
    assert np.allclose(s_sum, d.shape[1] * s)


def test_variable_draft_lengths():
    w = _weights()
    p, d = _ids(K=3, T=6)
    lens = np.array([6, 2, 4])
    lps, s = O.score_drafts(w, CFG, p, d, draft_lens=lens)
    for k in range(3):
        ref = O.token_logprobs(w, CFG, p, d[k, : lens[k]])
        assert np.allclose(lps[k, : lens[k]], ref) and np.all(lps[k, lens[k]:] == 0)
        assert math.isclose(s[k], -ref.mean())


# ---------------------------------------------------------------- rotary embedding
def test_rope_textbook_properties():
    rng = np.random.default_rng(2)
    x = rng.normal(size=(5, 3, 8))
    pos = np.array([0, 1, 2, 10, 500])
    y = O.rope_rotate_half(x, pos, 10000.0)
    assert np.array_equal(y[0], x[0])                                   # position 0: identity
    assert np.allclose((y ** 2).sum(-1), (x ** 2).sum(-1))              # a rotation
    # hd = 2, angle = pos * theta^0 = pos: quarter turn sends (a, b) -> (-b, a)
    q = O.rope_rotate_half(np.array([[[3.0, 4.0]]]), np.array([1]), 10000.0)
    assert np.allclose(q, [[[3 * math.cos(1) - 4 * math.sin(1), 4 * math.cos(1) + 3 * math.sin(1)]]])
    # relative-position property: <R_a q, R_b k> depends on a - b only
    qv, kv = rng.normal(size=(1, 1, 8)), rng.normal(size=(1, 1, 8))
    def dot(a, b):
        return float((O.rope_rotate_half(qv, np.array([a]), 1e4) * O.rope_rotate_half(kv, np.array([b]), 1e4)).sum())
    assert math.isclose(dot(7, 3), dot(104, 100), rel_tol=1e-12)
    assert not math.isclose(dot(7, 3), dot(3, 7), rel_tol=1e-6)
    # complex form: (x_i + i x_{i+h}) * exp(i pos theta^(-2i/hd))
    half = 4
    zc = (x[..., :half] + 1j * x[..., half:]) * np.exp(
        1j * pos[:, None, None] * (10000.0 ** (-2.0 * np.arange(half) / 8))[None, None, :])
    assert np.allclose(y, np.concatenate([zc.real, zc.imag], -1), rtol=0, atol=1e-12)


# ---------------------------------------------------------------- independent library formulation
def _torch_reference_logprobs(w, cfg, prefix, draft):
    t = lambda a: torch.from_numpy(np.asarray(a)).double()
    ids = torch.from_numpy(np.concatenate([prefix, draft]).astype(np.int64))
    n, nq, nkv, hd = len(ids), cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    h = F.embedding(ids, t(w["tok_embed"]))
    freqs = torch.polar(torch.ones(n, hd // 2, dtype=torch.float64),
                        torch.arange(n).double()[:, None]
                        * cfg.rope_theta ** (-torch.arange(0, hd, 2).double() / hd)[None, :])

    def rot(x):                       # x: [n, H, hd]
        xc = torch.complex(x[..., : hd // 2], x[..., hd // 2:]) * freqs[:, None, :]
        return torch.cat([xc.real, xc.imag], -1)

    for l in range(len(w["wqkv"])):
        a = F.rms_norm(h, (cfg.d_model,), t(w["attn_norm"][l]), cfg.rms_eps)
        q, k, v = F.linear(a, t(w["wqkv"][l])).split([nq * hd, nkv * hd, nkv * hd], -1)
        q, k, v = rot(q.view(n, nq, hd)), rot(k.view(n, nkv, hd)), v.view(n, nkv, hd)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                           v.transpose(0, 1)[None], is_causal=True, enable_gqa=True)
        h = h + F.linear(o[0].transpose(0, 1).reshape(n, nq * hd), t(w["wo"][l]))
        b = F.rms_norm(h, (cfg.d_model,), t(w["ffn_norm"][l]), cfg.rms_eps)
        g, u = F.linear(b, t(w["w_gate_up"][l])).chunk(2, -1)
        h = h + F.linear(F.silu(g) * u, t(w["w_down"][l]))
    z = F.linear(F.rms_norm(h, (cfg.d_model,), t(w["final_norm"]), cfg.rms_eps), t(w["lm_head"]))
    lsm = F.log_softmax(z, -1)
    P, T = len(prefix), len(draft)
    return lsm[torch.arange(P - 1, P - 1 + T), torch.from_numpy(draft.astype(np.int64))].numpy()


@pytest.mark.parametrize("cfg", [CFG, ModelConfig(3, 64, 8, 8, 8, 96, 80, "fp32"),
                                 ModelConfig(2, 48, 6, 1, 8, 64, 64, "bf16")])
def test_forward_matches_library_formulation(cfg):
    w = _weights(cfg, seed=13) if cfg.dtype == "fp32" else \
        {k: ([t.float().numpy() for t in v] if isinstance(v, list) else v.float().numpy())
         for k, v in make_weights(cfg, 13).items()}
    p, d = _ids(cfg, P=11, K=2, T=7)
    for k in range(2):
        got = O.token_logprobs(w, cfg, p, d[k])
        ref = _torch_reference_logprobs(w, cfg, p, d[k])
        assert np.allclose(got, ref, rtol=0, atol=1e-11)


def test_generator_is_device_independent_and_scaled():
    w1 = make_weights(CFG, 5)
    w2 = make_weights(CFG, 5)
    assert torch.equal(w1["wqkv"][1], w2["wqkv"][1])
    assert not torch.equal(w1["wqkv"][0], w1["wqkv"][1])
    assert abs(float(w1["tok_embed"].std()) - 1.0) < 0.05
    assert abs(float(w1["wqkv"][0].std()) - 1 / math.sqrt(CFG.d_model)) < 0.02
    wb = make_weights(ModelConfig(2, 32, 4, 2, 8, 48, 50, "bf16"), 5)
    assert wb["lm_head"].dtype == torch.bfloat16 and wb["final_norm"].dtype == torch.float32
    assert torch.equal(wb["lm_head"], w1["lm_head"].to(torch.bfloat16))


# ---- greedy continuation ("Target Model Sampling") ---------------------------------------------------------------

def test_greedy_continuation_is_the_argmax_chain_of_the_scored_distribution():
    """Two pins that do not re-use the function's own loop: (i) every generated token has the largest log-probability
    that token_logprobs assigns at its position (checked against every other token of a small vocabulary);
    (ii) the continuation does not depend on how the context is split into "prefix" and "draft"."""
    cfg = ModelConfig(2, 48, 4, 2, 12, 80, 37, "fp32")
    w = weights_to_numpy(make_weights(cfg, seed=11, device="cpu"))
    prefix = np.array([3, 1, 4, 1, 5, 9, 2, 6]); draft = np.array([5, 3, 5])
    toks, margins = O.greedy_continuation(w, cfg, prefix, draft, 4)
    assert toks.shape == (4,) and np.all(margins >= 0)
    ctx = np.concatenate([prefix, draft])
    for t in range(4):
        lp_best = O.token_logprobs(w, cfg, np.concatenate([ctx, toks[:t]]), toks[t:t + 1])[0]
        for other in range(cfg.vocab):
            lp = O.token_logprobs(w, cfg, np.concatenate([ctx, toks[:t]]), np.array([other]))[0]
            assert lp <= lp_best + 1e-12
    toks2, _ = O.greedy_continuation(w, cfg, ctx[:5], ctx[5:], 4)
    assert np.array_equal(toks, toks2)
    # a longer request extends a shorter one
    toks6, _ = O.greedy_continuation(w, cfg, prefix, draft, 6)
    assert np.array_equal(toks6[:4], toks)


def test_sampled_continuation_follows_the_scored_distribution():
    """Pins that do not re-use the function's loop: (i) over a fine grid of uniforms the first sampled token hits
    every token with the frequency token_logprobs assigns it (temperature 1); (ii) temperature -> 0 reproduces the
    greedy chain; (iii) u = 0 gives token 0, u -> 1 the last token with non-zero mass."""
    cfg = ModelConfig(1, 32, 2, 1, 16, 48, 11, "fp32")
    w = weights_to_numpy(make_weights(cfg, seed=3, device="cpu"))
    prefix = np.array([1, 2, 3, 4]); draft = np.array([5, 6])
    ctx = np.concatenate([prefix, draft])
    n = 4000
    us = (np.arange(n) + 0.5) / n
    first = np.array([O.sampled_continuation(w, cfg, prefix, draft, [u], 1.0)[0][0] for u in us])
    freq = np.bincount(first, minlength=cfg.vocab) / n
    p = np.exp([O.token_logprobs(w, cfg, ctx, np.array([v]))[0] for v in range(cfg.vocab)])
    assert abs(p.sum() - 1) < 1e-12 and np.abs(freq - p).max() <= 1.0 / n + 1e-12
    assert np.all(np.diff(first) >= 0)                                   # inverse CDF is monotone in u
    g, _ = O.greedy_continuation(w, cfg, prefix, draft, 3)
    t, _ = O.sampled_continuation(w, cfg, prefix, draft, [0.3, 0.9, 0.01], 1e-4)
    assert np.array_equal(g, t)
    assert O.sampled_continuation(w, cfg, prefix, draft, [0.0], 1.0)[0][0] == 0
    assert O.sampled_continuation(w, cfg, prefix, draft, [1.0 - 1e-16], 1.0)[0][0] == cfg.vocab - 1


def test_next_token_cdf_is_the_running_sum_of_the_scored_distribution():
    """The CDF helper against token_logprobs (not against its own softmax): its increments are the probabilities the
    scoring path assigns, at temperature tau they are proportional to p^(1/tau), and the token sampled_continuation
    draws for u is the one whose interval (cdf[v - 1], cdf[v]] holds u."""
    cfg = ModelConfig(1, 32, 2, 1, 16, 48, 11, "fp32")
    w = weights_to_numpy(make_weights(cfg, seed=3, device="cpu"))
    prefix = np.array([1, 2, 3, 4]); draft = np.array([5, 6])
    ctx = np.concatenate([prefix, draft])
    p = np.exp([O.token_logprobs(w, cfg, ctx, np.array([v]))[0] for v in range(cfg.vocab)])
    cdf = O.next_token_cdf(w, cfg, ctx, 1.0)
    assert cdf.shape == (cfg.vocab,) and abs(cdf[-1] - 1.0) < 1e-15 and np.all(np.diff(cdf) > 0)
    assert np.abs(np.diff(np.concatenate([[0.0], cdf])) - p).max() < 1e-12
    tau = 0.37
    q = p ** (1.0 / tau)
    assert np.abs(np.diff(np.concatenate([[0.0], O.next_token_cdf(w, cfg, ctx, tau)])) - q / q.sum()).max() < 1e-12
    for u in (0.0, 0.013, 0.25, 0.5, 0.77, 0.999):
        v = int(O.sampled_continuation(w, cfg, prefix, draft, [u], 1.0)[0][0])
        lo = cdf[v - 1] if v > 0 else 0.0
        assert (lo < u <= cdf[v]) or (u == 0.0 and v == 0)


def test_end_of_sequence_freezes_a_continuation():
    """With an end token the chain is the unconstrained chain up to and including the first occurrence of that token
    and the token itself afterwards; a token that never occurs changes nothing."""
    cfg = ModelConfig(2, 48, 4, 2, 12, 80, 37, "fp32")
    w = weights_to_numpy(make_weights(cfg, seed=11, device="cpu"))
    prefix = np.array([3, 1, 4, 1, 5, 9, 2, 6]); draft = np.array([5, 3, 5])
    free, _ = O.greedy_continuation(w, cfg, prefix, draft, 6)
    for s in range(6):
        eos = int(free[s])
        first = int(np.argmax(free == eos))                 # the token may already occur before step s
        got, m = O.greedy_continuation(w, cfg, prefix, draft, 6, eos_id=eos)
        assert np.array_equal(got[:first + 1], free[:first + 1]) and np.all(got[first + 1:] == eos)
        assert np.all(np.isinf(m[first + 1:])) and np.all(np.isfinite(m[:first + 1]))
    absent = next(v for v in range(cfg.vocab) if v not in set(free.tolist()))
    assert np.array_equal(O.greedy_continuation(w, cfg, prefix, draft, 6, eos_id=absent)[0], free)
    us = [0.3, 0.9, 0.01, 0.5, 0.7]
    sfree, _ = O.sampled_continuation(w, cfg, prefix, draft, us, 1.0)
    eos = int(sfree[1]); first = int(np.argmax(sfree == eos))
    sgot, sl = O.sampled_continuation(w, cfg, prefix, draft, us, 1.0, eos_id=eos)
    assert np.array_equal(sgot[:first + 1], sfree[:first + 1]) and np.all(sgot[first + 1:] == eos) and np.all(np.isinf(sl[first + 1:]))
