"""End-to-end parity of atts_score_drafts with the oracle (K independent fp64 causal forwards)."""
import numpy as np
import pytest
import torch

from oracle import atts_oracle as O
from synth import WORKLOADS, ModelConfig, make_token_ids, make_weights
from util import announce, dev, weights_to_numpy, ws

pytestmark = pytest.mark.gpu

TOL = {"fp32": 1e-4, "bf16": 2e-2}      # absolute, per-token log-prob


def _run_gpu(A, cfg, w_dev, prefix, drafts, lens=None, mode=0, want_lp=True):
    model = A.Model(cfg, w_dev)
    K, T = drafts.shape
    lp = torch.full((K, T), float("nan"), dtype=torch.float32, device="cuda") if want_lp else None
    sc = torch.full((K,), float("nan"), dtype=torch.float32, device="cuda")
    wsp = ws(A.atts_workspace_bytes(model, len(prefix), K, T))
    A.atts_score_drafts(model, dev(prefix), dev(drafts), None if lens is None else dev(lens), mode, lp, sc, wsp)
    torch.cuda.synchronize()
    flag = A.atts_model_check(model)
    return (None if lp is None else lp.cpu().numpy()), sc.cpu().numpy(), flag


def _case(cfg, P, K, T, seed, n_layers=None):
    w_dev = make_weights(cfg, seed, device="cuda", n_layers=n_layers)
    prefix, drafts = make_token_ids(cfg.vocab, P, K, T, seed)
    return w_dev, prefix.numpy(), drafts.numpy()


def test_generator_is_identical_on_cpu_and_gpu():
    cfg = ModelConfig(1, 64, 4, 2, 16, 96, 300, "bf16")
    a, b = make_weights(cfg, 9, "cpu"), make_weights(cfg, 9, "cuda")
    for k in a:
        for x, y in zip(a[k] if isinstance(a[k], list) else [a[k]], b[k] if isinstance(b[k], list) else [b[k]]):
            assert torch.equal(x, y.cpu()), k


@pytest.mark.parametrize("mode", [O.MEAN_NLL, O.SUM_NLL])
def test_tiny_workload_fp32(mode):
    import paper_2509_15148_amd as A
    wl = WORKLOADS["tiny"]
    announce("score tiny fp32 mode", mode)
    w_dev, prefix, drafts = _case(wl.model, wl.P, wl.K, wl.T, wl.seed)
    lp, sc, flag = _run_gpu(A, wl.model, w_dev, prefix, drafts, mode=mode)
    ref_lp, ref_s = O.score_drafts(weights_to_numpy(w_dev), wl.model, prefix, drafts, mode=mode)
    assert flag == 0
    assert np.abs(lp - ref_lp).max() <= TOL["fp32"], np.abs(lp - ref_lp).max()
    assert np.allclose(sc, ref_s, rtol=0, atol=TOL["fp32"] * (wl.T if mode == O.SUM_NLL else 1))


@pytest.mark.parametrize("cfg,P,K,T", [
    (ModelConfig(2, 256, 4, 2, 128, 520, 2003, "bf16"), 70, 3, 45),     # MFMA attention, ragged everywhere
    (ModelConfig(3, 128, 8, 2, 16, 264, 777, "bf16"), 33, 5, 9),        # simple attention in bf16
    (ModelConfig(1, 72, 6, 6, 12, 40, 100, "fp32"), 1, 1, 1),           # smallest call
    (ModelConfig(2, 96, 4, 1, 24, 200, 515, "fp32"), 19, 4, 23),
])
def test_small_models_ragged_shapes(cfg, P, K, T):
    import paper_2509_15148_amd as A
    announce("score small", cfg, P, K, T)
    w_dev, prefix, drafts = _case(cfg, P, K, T, seed=P * 1000 + K)
    lp, sc, flag = _run_gpu(A, cfg, w_dev, prefix, drafts)
    ref_lp, ref_s = O.score_drafts(weights_to_numpy(w_dev), cfg, prefix, drafts)
    assert flag == 0
    assert np.abs(lp - ref_lp).max() <= TOL[cfg.dtype], np.abs(lp - ref_lp).max()
    assert np.abs(sc - ref_s).max() <= TOL[cfg.dtype]
    # scores only (token_logprobs = NULL) gives the same scores, bit for bit: calls with this few rows split the K range
    # of some projections over workgroups, whose partial sums are added in a fixed order
    _, sc2, _ = _run_gpu(A, cfg, w_dev, prefix, drafts, want_lp=False)
    assert np.array_equal(sc, sc2)


def test_variable_draft_lengths_and_padding_ids():
    import paper_2509_15148_amd as A
    cfg = ModelConfig(2, 256, 4, 2, 128, 512, 1000, "bf16")
    announce("score draft_lens")
    w_dev, prefix, drafts = _case(cfg, 40, 4, 30, seed=5)
    lens = np.array([30, 1, 17, 29], dtype=np.int32)
    padded = drafts.copy()
    for k in range(4):
        padded[k, lens[k]:] = -12345                      # garbage ids in the padding are ignored
    lp, sc, flag = _run_gpu(A, cfg, w_dev, prefix, padded, lens=lens)
    ref_lp, ref_s = O.score_drafts(weights_to_numpy(w_dev), cfg, prefix, drafts, draft_lens=lens)
    assert flag == 0
    assert np.abs(lp - ref_lp).max() <= TOL["bf16"]
    for k in range(4):
        assert np.all(lp[k, lens[k]:] == 0)
    assert np.abs(sc - ref_s).max() <= TOL["bf16"]


def test_out_of_range_token_id_sets_the_flag_and_does_not_fault():
    import paper_2509_15148_amd as A
    cfg = ModelConfig(1, 64, 4, 2, 16, 96, 50, "fp32")
    announce("score bad id")
    w_dev, prefix, drafts = _case(cfg, 6, 2, 4, seed=1)
    bad = drafts.copy()
    bad[1, 2] = 50
    lp, sc, flag = _run_gpu(A, cfg, w_dev, prefix, bad)
    assert flag == 1 and np.all(np.isfinite(lp))
    lp, sc, flag = _run_gpu(A, cfg, w_dev, prefix, drafts)
    assert flag == 0


def test_workspace_and_argument_errors():
    import paper_2509_15148_amd as A
    cfg = ModelConfig(1, 64, 4, 2, 16, 96, 50, "fp32")
    w_dev, prefix, drafts = _case(cfg, 6, 2, 4, seed=1)
    model = A.Model(cfg, w_dev)
    need = A.atts_workspace_bytes(model, 6, 2, 4)
    sc = torch.empty(2, device="cuda")
    with pytest.raises(A.AttsError) as e:
        A.atts_score_drafts(model, dev(prefix), dev(drafts), None, 0, None, sc, ws(need)[: need - 256])
    assert e.value.code == A.ERR_WORKSPACE
    with pytest.raises(A.AttsError) as e:
        A.atts_score_drafts(model, dev(prefix), dev(drafts), None, 5, None, sc, ws(need))
    assert e.value.code == A.ERR_INVALID_ARG
    with pytest.raises(A.AttsError) as e:
        A.atts_score_drafts(model, dev(prefix)[:0], dev(drafts), None, 0, None, sc, ws(need))
    assert e.value.code == A.ERR_INVALID_ARG


def _full_width_case(name, n_layers, k_sample, shape=None):
    """GPU: the whole workload (all K drafts) in the benchmark's launch configuration (or the same model at
    another (P, K, T)).  Oracle: the drafts in `k_sample` (an index, a list of indices or "all"), each alone as one
    plain causal sequence; every draft's first token against the prediction from the last prefix position."""
    import paper_2509_15148_amd as A
    wl = WORKLOADS[name]
    cfg = wl.model
    P, K, T = shape if shape else (wl.P, wl.K, wl.T)
    sample = list(range(K)) if k_sample == "all" else ([k_sample] if isinstance(k_sample, int) else list(k_sample))
    announce("score full width", name, "layers", n_layers, "shape", (P, K, T), "sample drafts", sample)
    w_dev, prefix, drafts = _case(cfg, P, K, T, wl.seed, n_layers=n_layers)
    lp, sc, flag = _run_gpu(A, cfg, w_dev, prefix, drafts)
    assert flag == 0 and np.all(np.isfinite(lp)) and np.all(lp <= 0)
    if shape is not None:      # run-to-run bit-stability, also where projections split their K range over workgroups
        lp2, sc2, _ = _run_gpu(A, cfg, w_dev, prefix, drafts)
        assert np.array_equal(lp, lp2) and np.array_equal(sc, sc2)
    w_np = weights_to_numpy(w_dev)
    del w_dev
    torch.cuda.empty_cache()
    worst = 0.0
    for k in sample:
        ref = O.token_logprobs(w_np, cfg, prefix, drafts[k])
        err = np.abs(lp[k] - ref).max()
        worst = max(worst, float(err))
        assert err <= TOL["bf16"], (k, err)
        assert abs(sc[k] - O.conformity_score(ref)) <= TOL["bf16"], k
    print(f"[score full width {name} L={n_layers} {(P, K, T)}] max |dlogp| over drafts {sample} = {worst:.3e}", flush=True)
    # all drafts share the prediction of their first token from the last prefix position
    first = O.log_softmax(O.logits_from_hidden(w_np, cfg, O.decoder_hidden(w_np, cfg, prefix)[-1:]))[0]
    assert np.abs(lp[:, 0] - first[drafts[:, 0]]).max() <= TOL["bf16"]


@pytest.mark.timeout(900)
def test_7b_shape_two_layer_slice():
    """The benchmark's launch configuration at 7B width, two layers: EVERY one of the 16 drafts element by element."""
    _full_width_case("7b", n_layers=2, k_sample="all")


@pytest.mark.parametrize("shape", [(16, 16, 8), (300, 5, 67), (1, 2, 3), (700, 3, 100)])
def test_7b_width_few_and_ragged_rows(shape):
    """Row counts that are not whole 256-row tiles, at full model width: the decode-like shape that bench.py
    times (144 rows: projections with few tiles split their K range over several workgroups), a ragged
    multi-tile one, a handful of rows, and 1000 rows (four tile rows, still few enough tiles to split K).  All drafts
    are compared, and a second run must reproduce the first bit for bit."""
    _full_width_case("7b", n_layers=2, k_sample="all", shape=shape)


@pytest.mark.timeout(900)
def test_7b_full_model_sampled_draft():
    """The 7B-class workload exactly as bench.py runs it (28 layers, K = 16 drafts of 256 tokens after a
    512-token prefix); the oracle scores one sampled draft as a plain causal sequence (~1 minute of CPU)."""
    _full_width_case("7b", n_layers=None, k_sample=11)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name", ["32b", "70b"])
def test_large_models_two_layer_slice(name):
    """Full width, full row count (34,816 / 9,216 rows: 64-bit offsets in the FFN activation), two layers (the
    residual epilogue -> norm -> next layer hand-off at these widths); the oracle scores the first and the last
    draft (the last one ends in the last, ragged row tile)."""
    K = WORKLOADS[name].K
    _full_width_case(name, n_layers=2, k_sample=(3, K - 1))
