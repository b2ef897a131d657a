"""Plain fp64 CPU oracle for the ATTS verification / conformal hot path.

TEST INFRASTRUCTURE ONLY.  This module is the slow, obviously-correct statement of what
the path computes, written out from the paper's definitions in numpy float64.  Only the
test-suite, the smoke check and the benchmark's CPU-baseline leg may import it; the
product (the HIP library and its Python binding) never does, and shares no code with it.

What is defined here, and from where:

  * target-model verification of a draft continuation given the prompt prefix
    (Sec. "How to perform rejection sampling via conformal prediction", paragraph
    "Verification"): the logits of the target model for every draft token, teacher-forced.
    The paper fixes no architecture; the decoder below (pre-norm, RMSNorm, rotate-half
    RoPE, grouped-query causal attention, SwiGLU FFN, untied LM head, no biases) is the
    reading used throughout this repository.
  * the unnormalised conformity score  s = -l(X, Y)  (Sec. "Q2", paragraph "Online
    Calibration", the unnumbered equation defining s_xi^k): here the negative
    log-likelihood of the draft under the target, MEAN over tokens (log-perplexity) or SUM.
  * the marginal conformal p-value (Eq. "p-value" / Proposition 1):
        p = (#{calibration scores s_i^j : s_test <= s_i^j} + 1) / (n m + 1)
  * the accept rule  p > alpha  (Eq. "prediction_set"); reject iff p <= alpha, the event
    Proposition 1 bounds by alpha.
  * the classic conformal quantile (Sec. "Preliminary", Eq. "quantile"): the
    ceil((N+1)(1-alpha))-th smallest calibration score.
  * ordinal classes from several ascending levels alpha_1 < ... < alpha_n:
        class = #{l : p <= alpha_l}
    (0 = accept; with two levels 1 = resample, 2 = target fallback).  This multi-level
    rule is a generalisation of the paper's single-alpha accept/reject, not a formula the
    paper prints.
  * online calibration (paragraph "Online Calibration"): the calibration multiset grows
    by the scores of newly pre-sampled outputs; every rank refers to the multiset as it
    stands at that moment.
  * target-model continuation of a rejected candidate (paragraph "Target Model Sampling"): greedy
    (the arg max of the target's next-token logits, token by token) or sampled from the
    temperature-scaled softmax by inverse CDF, the uniform draws being inputs.
  * conditional coverage (same paragraph, last sentence; Proposition 2): the same rank,
    p-value and classes, but each input's candidates are compared with that input's own
    calibration scores only.
  * the classic, synchronous pipeline the method is measured against (Sec. "Preliminary",
    "Classic Setup"): scores normalised over the m candidates of an input (Eq. "softmax"),
    one global threshold tau = an order statistic of ALL normalised calibration scores
    (Eq. "quantile") and the prediction set {k : s^k >= tau} (Eq. "pred_set").  No candidate of
    an input can be decided before all m of its scores are there: the synchronisation the
    asynchronous arithmetic intensity of Sec. "Q1" charges as T_s.

Pins (see tests/test_oracle_*.py): closed forms for the log-softmax and for degenerate
models, causal-prefix invariances of the forward pass, the uniform distribution of
p-values for distinct scores and the tie formula of Proposition 1's proof, exact
enumeration of the coverage guarantee (marginal, and per input for the conditional
variant: Proposition 2's uniform law), equivalence of the rank rule with the classic
quantile rule, hand-worked fixtures under tests/golden/, and for the classic pipeline the
logistic closed form of a two-candidate softmax, shift invariance, the brute-force
definition of an order statistic and the set size floor(alpha (N + 1)) on distinct scores.  The decoder forward has no
paper-printed numeric example: beyond the invariants and closed forms it is
"parity unpinned" to any external numeric source.
"""
from __future__ import annotations

import math
from typing import Optional, Sequence

import numpy as np

F64 = np.float64

MEAN_NLL = 0
SUM_NLL = 1


# --------------------------------------------------------------------------------------
# Target model forward (the "Verification" step), fp64, one token sequence at a time
# --------------------------------------------------------------------------------------

def _w(a) -> np.ndarray:
    """Stored weight values widened to float64 (no other rounding anywhere)."""
    return np.asarray(a, dtype=F64)


def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """x * gain / sqrt(mean(x^2) + eps), over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x * _w(gain) / np.sqrt(ms + eps)


def rope_rotate_half(x: np.ndarray, positions: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding, rotate-half pairing.  x: [n, heads, hd]; positions: [n].

    Pair (i, i + hd/2), 0 <= i < hd/2, is rotated by angle  pos * theta^(-2 i / hd).
    """
    n, _, hd = x.shape
    half = hd // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=F64) / hd)
    ang = positions.astype(F64)[:, None] * inv_freq[None, :]          # [n, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def decoder_hidden(weights, cfg, ids: np.ndarray) -> np.ndarray:
    """Residual stream after the last layer for one plain causal sequence.  ids: [n].

    cfg needs: n_q_heads, n_kv_heads, head_dim, d_ffn, rope_theta, rms_eps.
    weights: dict as produced by synth.make_weights (any float dtype; widened here);
    the number of layers is len(weights["wqkv"]).
    """
    nq, nkv, hd = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    F = cfg.d_ffn
    group = nq // nkv
    n = len(ids)
    pos = np.arange(n)
    h = _w(weights["tok_embed"][np.asarray(ids, dtype=np.int64)])     # [n, d]
    causal = np.tril(np.ones((n, n), dtype=bool))
    for l in range(len(weights["wqkv"])):
        a = rmsnorm(h, weights["attn_norm"][l], cfg.rms_eps)
        qkv = a @ _w(weights["wqkv"][l]).T                            # [n, (nq+2nkv) hd]
        q = qkv[:, : nq * hd].reshape(n, nq, hd)
        k = qkv[:, nq * hd: (nq + nkv) * hd].reshape(n, nkv, hd)
        v = qkv[:, (nq + nkv) * hd:].reshape(n, nkv, hd)
        q = rope_rotate_half(q, pos, cfg.rope_theta)
        k = rope_rotate_half(k, pos, cfg.rope_theta)
        ctx = np.empty((n, nq, hd), dtype=F64)
        for j in range(nq):
            kv = j // group
            sc = (q[:, j, :] @ k[:, kv, :].T) / math.sqrt(hd)         # [n, n]
            sc = np.where(causal, sc, -np.inf)
            sc = sc - sc.max(axis=-1, keepdims=True)
            pr = np.exp(sc)
            pr /= pr.sum(axis=-1, keepdims=True)
            ctx[:, j, :] = pr @ v[:, kv, :]
        h = h + ctx.reshape(n, nq * hd) @ _w(weights["wo"][l]).T
        b = rmsnorm(h, weights["ffn_norm"][l], cfg.rms_eps)
        gu = b @ _w(weights["w_gate_up"][l]).T                        # [n, 2F]: gate | up
        h = h + (silu(gu[:, :F]) * gu[:, F:]) @ _w(weights["w_down"][l]).T
    return h


def logits_from_hidden(weights, cfg, h: np.ndarray) -> np.ndarray:
    """z = W_lm . RMSNorm(h; g_final).  h: [n, d] -> [n, V]."""
    return rmsnorm(h, weights["final_norm"], cfg.rms_eps) @ _w(weights["lm_head"]).T


def log_softmax(z: np.ndarray) -> np.ndarray:
    """Row-wise  z - log sum_v exp(z_v)  (max-shifted)."""
    m = z.max(axis=-1, keepdims=True)
    return z - (m + np.log(np.exp(z - m).sum(axis=-1, keepdims=True)))


def token_logprobs(weights, cfg, prefix_ids, draft_ids) -> np.ndarray:
    """log q_t(y_t | x, y_<t) for every token of ONE draft continuation.  -> [T].

    The sequence [x_0..x_{P-1}, y_0..y_{T-1}] is run causally; the logits at position i
    predict the token at position i+1, so y_t is read from position P-1+t.
    """
    prefix_ids = np.asarray(prefix_ids, dtype=np.int64)
    draft_ids = np.asarray(draft_ids, dtype=np.int64)
    P, T = len(prefix_ids), len(draft_ids)
    h = decoder_hidden(weights, cfg, np.concatenate([prefix_ids, draft_ids]))
    lsm = log_softmax(logits_from_hidden(weights, cfg, h[P - 1: P - 1 + T]))
    return lsm[np.arange(T), draft_ids]


def greedy_continuation(weights, cfg, prefix_ids, draft_ids, n_new: int, eos_id=None):
    """Target-model continuation of one candidate (Sec. "How to perform rejection sampling via conformal
    prediction", paragraph "Target Model Sampling"): the candidate's draft is kept as a prefix and the target model
    generates n_new more tokens.  Decoding here is greedy: every new token is the arg max of the target's
    next-token logits given everything before it (first index on exact ties, as numpy's argmax).

    Returns (tokens [n_new] int64, margins [n_new] float64) where margins[t] is the gap between the best and the
    second-best logit at step t (how close the decision was).  With eos_id, a candidate that has produced that
    token has ended: the rest of its fixed-size output repeats eos_id (margin inf: nothing was decided there).
    """
    ctx = [int(t) for t in np.concatenate([np.asarray(prefix_ids), np.asarray(draft_ids)])]
    toks, margins = [], []
    for _ in range(n_new):
        if eos_id is not None and toks and toks[-1] == eos_id:
            toks.append(int(eos_id))
            margins.append(np.inf)
            continue
        h = decoder_hidden(weights, cfg, np.asarray(ctx, dtype=np.int64))
        z = logits_from_hidden(weights, cfg, h[-1:])[0]
        best = int(np.argmax(z))
        second = np.partition(z, -2)[-2]
        toks.append(best)
        margins.append(float(z[best] - second))
        ctx.append(best)
    return np.asarray(toks, dtype=np.int64), np.asarray(margins, dtype=F64)


def next_token_cdf(weights, cfg, context_ids, temperature: float) -> np.ndarray:
    """Cumulative distribution, in vocabulary order, of the target's next token after `context_ids` under
    softmax(logits / temperature) (paragraph "Target Model Sampling"): cdf[v] = P(token <= v), cdf[-1] = 1.
    Token v owns the interval (cdf[v - 1], cdf[v]] of a uniform draw (cdf[-1] read as 0)."""
    h = decoder_hidden(weights, cfg, np.asarray(context_ids, dtype=np.int64))
    z = logits_from_hidden(weights, cfg, h[-1:])[0] / float(temperature)
    c = np.cumsum(np.exp(z - z.max()))
    return c / c[-1]


def sampled_continuation(weights, cfg, prefix_ids, draft_ids, uniforms, temperature: float, eos_id=None):
    """Target-model continuation by sampling (paragraph "Target Model Sampling"): token t is drawn from
    softmax(logits / temperature) of the target given everything before it.  The randomness is an input: with
    u = uniforms[t] in [0, 1) the token is the first index v (vocabulary order) whose cumulative probability
    reaches u, i.e. inverse-CDF sampling.

    Returns (tokens [n] int64, slack [n] float64): slack[t] is the distance, in probability, from u to the nearer
    end of the chosen token's CDF interval (how close the draw was to picking a neighbour).  eos_id as in
    greedy_continuation (slack inf after the end; the uniforms of those positions are not used).
    """
    ctx = [int(t) for t in np.concatenate([np.asarray(prefix_ids), np.asarray(draft_ids)])]
    toks, slack = [], []
    for u in np.asarray(uniforms, dtype=F64):
        if eos_id is not None and toks and toks[-1] == eos_id:
            toks.append(int(eos_id))
            slack.append(np.inf)
            continue
        h = decoder_hidden(weights, cfg, np.asarray(ctx, dtype=np.int64))
        z = logits_from_hidden(weights, cfg, h[-1:])[0] / float(temperature)
        p = np.exp(z - z.max())
        cdf = np.cumsum(p)
        target = u * cdf[-1]
        v = int(np.searchsorted(cdf, target, side="left"))
        v = min(v, len(cdf) - 1)
        lo = cdf[v - 1] if v > 0 else 0.0
        toks.append(v)
        slack.append(float(min(target - lo, cdf[v] - target) / cdf[-1]))
        ctx.append(v)
    return np.asarray(toks, dtype=np.int64), np.asarray(slack, dtype=F64)


def conformity_score(logprobs: np.ndarray, mode: int = MEAN_NLL) -> float:
    """s = -l(X, Y): negative log-likelihood of the draft; mean over its tokens or sum."""
    lp = np.asarray(logprobs, dtype=F64)
    total = -float(lp.sum())
    return total / len(lp) if mode == MEAN_NLL else total


def score_drafts(weights, cfg, prefix_ids, draft_ids, draft_lens=None, mode: int = MEAN_NLL):
    """K independent verifications.  draft_ids: [K, T_max]; draft_lens: [K] or None.

    Returns (logprobs [K, T_max] with 0 at padded positions, scores [K]).
    """
    draft_ids = np.asarray(draft_ids)
    K, T_max = draft_ids.shape
    lens = np.full(K, T_max) if draft_lens is None else np.asarray(draft_lens)
    lp = np.zeros((K, T_max), dtype=F64)
    s = np.zeros(K, dtype=F64)
    for k in range(K):
        t = int(lens[k])
        lp[k, :t] = token_logprobs(weights, cfg, prefix_ids, draft_ids[k, :t])
        s[k] = conformity_score(lp[k, :t], mode)
    return lp, s


# --------------------------------------------------------------------------------------
# Conformal layer: ranks, p-values, thresholds, ordinal classes, online calibration
# --------------------------------------------------------------------------------------

def rank_counts(cal: np.ndarray, test: np.ndarray) -> np.ndarray:
    """c[i] = #{j : test[i] <= cal[j]} -- the double sum of Eq. "p-value", as written.

    IEEE comparisons: a NaN on either side never counts; -0 == +0.
    """
    cal = np.asarray(cal, dtype=F64)
    test = np.asarray(test, dtype=F64)
    c = np.zeros(len(test), dtype=np.int64)
    for i, s in enumerate(test):
        c[i] = int(np.count_nonzero(s <= cal))
    return c


def rank_counts_sorted(cal: np.ndarray, test: np.ndarray) -> np.ndarray:
    """Same counts through a library sort + binary search (for sizes where the double
    sum takes minutes).  NaN calibration scores are dropped (they never satisfy <=);
    a NaN test score gets 0."""
    cal = np.asarray(cal, dtype=F64)
    test = np.asarray(test, dtype=F64)
    srt = np.sort(cal[~np.isnan(cal)])
    c = len(srt) - np.searchsorted(srt, test, side="left")
    return np.where(np.isnan(test), 0, c).astype(np.int64)


def p_values(counts: np.ndarray, n_cal: int) -> np.ndarray:
    """p = (c + 1) / (N + 1)."""
    return (np.asarray(counts, dtype=F64) + 1.0) / (n_cal + 1.0)


def reject_ranks(alphas: Sequence[float], n_cal: int) -> np.ndarray:
    """r_l = floor(alpha_l (N+1)), one binary64 multiply then floor.

    p <= alpha_l  <=>  c + 1 <= alpha_l (N+1)  <=>  c + 1 <= r_l   (c + 1 is an integer),
    so every decision is an integer comparison."""
    return np.array([math.floor(float(a) * float(n_cal + 1)) for a in alphas], dtype=np.int64)


def classify(counts: np.ndarray, ranks_r: np.ndarray) -> np.ndarray:
    """class = #{l : p <= alpha_l} = #{l : c + 1 <= r_l}; uint8."""
    c1 = np.asarray(counts, dtype=np.int64)[:, None] + 1
    return (c1 <= np.asarray(ranks_r, dtype=np.int64)[None, :]).sum(axis=1).astype(np.uint8)


def quantile_thresholds(cal: np.ndarray, ranks_r: np.ndarray) -> np.ndarray:
    """Q_l = the (N + 1 - r_l)-th smallest calibration score (1-indexed), i.e. the
    ceil((1 - alpha_l)(N + 1))-th order statistic of Eq. "quantile";  +inf when
    r_l = 0 (nothing can be rejected), -inf when r_l >= N + 1.

    A NaN calibration score is never ">=" anything, so it orders below every number
    here (and is returned as NaN if selected)."""
    cal = np.asarray(cal, dtype=F64)
    nan = np.isnan(cal)
    srt = np.concatenate([cal[nan], np.sort(cal[~nan])])
    n = len(srt)
    out = np.empty(len(ranks_r), dtype=F64)
    for l, r in enumerate(np.asarray(ranks_r, dtype=np.int64)):
        kth = n + 1 - int(r)
        out[l] = np.inf if kth > n else (-np.inf if kth < 1 else srt[kth - 1])
    return out


def conditional_classify(cal_sets, test_sets, alphas: Sequence[float]):
    """Conditional coverage (Sec. Q2, last sentence of "Online Calibration"; Proposition 2): the candidates of
    input xi are ranked against the calibration scores of the SAME input only.

    For every input xi with its own m_xi calibration scores and its test scores s:
        c = #{j : s <= cal_xi[j]},  p = (c + 1) / (m_xi + 1),  class = #{l : c + 1 <= floor(alpha_l (m_xi + 1))}.
    The comparison direction and the integer form of "p <= alpha" are those of the marginal rule; only the set
    compared against changes (and with it the normaliser: m_xi + 1, as in Proposition 2's uniform law).
    Returns three lists (counts int64, p binary64, classes uint8), one array per input.
    """
    assert len(cal_sets) == len(test_sets)
    counts, ps, classes = [], [], []
    for cal, test in zip(cal_sets, test_sets):
        cal = np.asarray(cal, dtype=F64)
        c = rank_counts(cal, np.asarray(test, dtype=F64))
        r = reject_ranks(alphas, len(cal))
        counts.append(c)
        ps.append(p_values(c, len(cal)))
        classes.append(classify(c, r))
    return counts, ps, classes


# --------------------------------------------------------------------------------------
# The classic (synchronous) pipeline: normalised scores, global quantile, prediction sets
# --------------------------------------------------------------------------------------

def classic_softmax_scores(nll: np.ndarray) -> np.ndarray:
    """Eq. "softmax": s[i, k] = exp(-l[i, k]) / sum_j exp(-l[i, j]) over the m candidates of input i.

    `nll` [n, m] holds l(X_i, Y_i^k) >= 0, the negative log-likelihood of candidate k (the unnormalised
    score of the asynchronous design), so s is the candidate's share of the likelihood mass of its input:
    larger = more likely.  The row minimum of l is subtracted from the row before exponentiating; the
    quotient is unchanged by it (numerator and denominator are both multiplied by exp(min l)) and rows with
    l in the thousands (SUM scores of long drafts) do not underflow to 0 / 0."""
    l = np.asarray(nll, dtype=F64)
    assert l.ndim == 2
    e = np.exp(-(l - l.min(axis=1, keepdims=True)))
    return e / e.sum(axis=1, keepdims=True)


def classic_threshold(cal_scores: np.ndarray, alpha: float) -> float:
    """Eq. "quantile": tau = the p-quantile of ALL N normalised calibration scores, p = ceil((N + 1)(1 - alpha)) / N,
    i.e. the k-th smallest of them with k = ceil((N + 1)(1 - alpha)) = N + 1 - floor(alpha (N + 1))
    (the floor taken of one binary64 product, the same integer the rank rule uses); +inf if k > N, -inf if k < 1.
    This is the global sort every turn of the synchronous design pays for."""
    s = np.sort(np.asarray(cal_scores, dtype=F64).ravel())
    n = len(s)
    k = n + 1 - math.floor(float(alpha) * float(n + 1))
    if k > n:
        return math.inf
    if k < 1:
        return -math.inf
    return float(s[k - 1])


def classic_prediction_sets(scores: np.ndarray, tau: float) -> np.ndarray:
    """Eq. "pred_set": C(X_i) = {k : s[i, k] >= tau}, returned as a uint8 membership mask shaped like `scores`."""
    return (np.asarray(scores, dtype=F64) >= tau).astype(np.uint8)


class CalibrationSet:
    """Append-only multiset of calibration scores (online calibration)."""

    def __init__(self):
        self.scores = np.zeros(0, dtype=F64)

    def append(self, new_scores) -> None:
        self.scores = np.concatenate([self.scores, np.asarray(new_scores, dtype=F64)])

    def __len__(self) -> int:
        return len(self.scores)

    def classify(self, test, alphas, brute_force: bool = True):
        """-> (counts int64 [M], p-values f64 [M], classes uint8 [M], thresholds f64 [n_alpha])."""
        rank = rank_counts if brute_force else rank_counts_sorted
        c = rank(self.scores, test)
        r = reject_ranks(alphas, len(self))
        return c, p_values(c, len(self)), classify(c, r), quantile_thresholds(self.scores, r)
