#!/usr/bin/env python3
"""Throughput of the ATTS hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input, inputs resident in
HBM: atts_score_drafts (prefix + K drafts through the target model, fused LM-head log-softmax-
gather, conformity scores) -> atts_classify_ordinal of the K fresh scores against the calibration
set -> atts_calibrate_online appending them.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 7b|32b|70b|tiny] [--layers L]
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "fp32": 157.3}     # MI355X dense peaks
HBM_PEAK_GBS = 8000.0

# HBM traffic of the dominant kernel (gate/up GEMM, 7B workload) per launch, from two rocprofv3 --pmc runs
# (FETCH_SIZE, then WRITE_SIZE), each scaled by what the same counter reads for a plain device copy of known
# size (--traffic-probe); see profiles/traffic_gemm_gate_up_7b.txt.  Valid only for the kernel source it was
# taken with: reported as null when the hash of csrc/gemm.hip differs.
MEASURED_TRAFFIC = {"gemm_sha256": "be847675f147059c48d5d5cdf77993c07690a2abac66844243b7e210c8fb4ade",
                    "workload": "7b", "bytes_per_launch": 1.753e9}


def measured_traffic(workload):
    import hashlib
    src = os.path.join(ROOT, "paper_2509_15148_amd", "csrc", "gemm.hip")
    sha = hashlib.sha256(open(src, "rb").read()).hexdigest()
    if workload == MEASURED_TRAFFIC["workload"] and sha == MEASURED_TRAFFIC["gemm_sha256"]:
        return MEASURED_TRAFFIC["bytes_per_launch"]
    return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_flops(cfg, P, K, T, n_layers):
    """Flops the method must perform (no padding, no masked-out triangle)."""
    rows, B = P + K * T, K * T
    d, hd, nq, nkv, F, V = cfg.d_model, cfg.head_dim, cfg.n_q_heads, cfg.n_kv_heads, cfg.d_ffn, cfg.vocab
    per_row = {
        "gemm_qkv": 2 * d * (nq + 2 * nkv) * hd,
        "gemm_o": 2 * nq * hd * d,
        "gemm_gate_up": 2 * d * 2 * F,
        "gemm_down": 2 * F * d,
    }
    fl = {k: v * rows * n_layers for k, v in per_row.items()}
    ctx = sum(i + 1 for i in range(P)) + K * sum(P + t + 1 for t in range(T))
    fl["attention"] = 4 * hd * nq * ctx * n_layers
    fl["lmhead"] = 2 * B * d * V
    fl["total"] = sum(fl.values())
    return fl


def cpu_baseline(cfg, wl, w_dev, prefix, drafts, n_layers_full, budget_layers):
    """The oracle, as it stands, on a bounded sample: ONE draft (P + T tokens) through the first
    `budget_layers` layers + the LM head, extrapolated to all layers by the layer count."""
    import numpy as np
    import torch
    from oracle import atts_oracle as O

    sub = {k: (v[:budget_layers] if isinstance(v, list) else v) for k, v in w_dev.items()}
    w_np = {k: ([t.float().cpu().numpy() for t in v] if isinstance(v, list) else v.float().cpu().numpy())
            for k, v in sub.items()}
    seq = np.concatenate([prefix, drafts[0]])
    t0 = time.perf_counter()
    h = O.decoder_hidden(w_np, cfg, seq)
    t1 = time.perf_counter()
    lsm = O.log_softmax(O.logits_from_hidden(w_np, cfg, h[wl.P - 1: wl.P - 1 + wl.T]))
    _ = lsm[np.arange(wl.T), drafts[0]]
    t2 = time.perf_counter()
    t_layers, t_head = t1 - t0, t2 - t1
    t_full = t_layers * n_layers_full / max(budget_layers, 1) + t_head
    whole = budget_layers == n_layers_full
    return {
        "value": wl.T / t_full, "unit": "tokens/s", "cores": torch.get_num_threads(), "kind": "oracle",
        "extrapolated": not whole,
        "sample": (f"numpy fp64 oracle, 1 of {wl.K} drafts ({wl.P}+{wl.T} tokens) through "
                   + (f"all {n_layers_full} layers ({t_layers:.1f} s) + LM head ({t_head:.1f} s); value = {wl.T} tokens / that time"
                      if whole else
                      f"{budget_layers} of {n_layers_full} layers ({t_layers:.1f} s) + LM head ({t_head:.1f} s); value = "
                      f"{wl.T} tokens / (layer time x {n_layers_full}/{budget_layers} + head time), an extrapolation by layer count")),
    }


def calibration_cpu_baseline(np, torch, n_cal, n_new, n_test, alphas, draw, steps, note):
    """The oracle's conformal layer on the calibration-only step: append n_new scores, then ranks (library sort + binary
    search form of Eq. "p-value"), classes and thresholds of n_test scores; wall time per step on the host cores."""
    from oracle import atts_oracle as O
    cs = O.CalibrationSet()
    cs.append(draw(n_cal, 1))
    new = [draw(n_new, 10 + i) for i in range(steps)]
    test = [draw(n_test, 100 + i) for i in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        cs.append(new[i])
        cs.classify(test[i], alphas, brute_force=False)
    dt = (time.perf_counter() - t0) / steps
    return {"value": n_test / dt, "unit": "decisions/s", "cores": torch.get_num_threads(), "kind": "oracle",
            "us_per_step": dt * 1e6, "sample": note}


def bench_calibration(A, torch, np, steps=16, scaled=False, cpu=True):
    """The calibration-only workload: 2^20 resident scores, then per step append 65,536 and classify 65,536 at
    two alpha levels.  scaled=True: the same step at an out-of-cache size (2^28 resident scores = 1 GiB of keys,
    2^24 appended and 2^24 classified per step), where the HBM roofline is the meaningful bound; its scores are
    drawn on the device (exp of a seeded normal)."""
    from synth import WORKLOADS, lognormal_scores
    wl = WORKLOADS["calib"]
    if scaled:
        n_cal, n_new, n_test = 1 << 28, 1 << 24, 1 << 24
        g = torch.Generator(device="cuda").manual_seed(wl.seed)
        draw = lambda n, _seed: torch.randn(n, device="cuda", generator=g).exp_()
    else:
        n_cal, n_new, n_test = wl.n_cal, wl.n_new, wl.n_test
        draw = lambda n, seed: torch.from_numpy(lognormal_scores(n, seed)).cuda()
    calib = A.Calib(n_cal + (2 * steps + 2) * n_new)
    A.atts_calibrate_online(calib, draw(n_cal, wl.seed))
    new = [draw(n_new, wl.seed + 1000 + i) for i in range(steps + 2)]
    test = [draw(n_test, wl.seed + 2000 + i) for i in range(steps + 2)]
    ranks = torch.empty(n_test, dtype=torch.int32, device="cuda")
    cls = torch.empty(n_test, dtype=torch.uint8, device="cuda")

    def step(i):
        A.atts_calibrate_online(calib, new[i])
        A.atts_classify_ordinal(calib, test[i], list(wl.alphas), ranks, None, cls, None)

    step(0)
    step(1)
    torch.cuda.synchronize()
    n0 = A.atts_calib_size(calib)
    t0 = time.perf_counter()
    for i in range(2, steps + 2):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    n_mid = n0 + n_new * steps / 2
    # per-kernel-group device times of the same steps again (HIP events on the launch stream)
    A.atts_profile_enable(True)
    for i in range(2, steps + 2):
        step(i)
    torch.cuda.synchronize()
    st = {name: A.atts_profile_read(A.STAGES.index(name))[0] / steps * 1e3 for name in ("calib_sort", "calib_merge", "classify")}
    A.atts_profile_enable(False)
    # decisions only (ranks = NULL): classes from the threshold form of the rule, no search per score; device time
    # from the library's events (at the small size a Python call costs more than the kernel)
    A.atts_classify_ordinal(calib, test[0], list(wl.alphas), None, None, cls, None)
    torch.cuda.synchronize()
    A.atts_profile_enable(True)
    for i in range(steps):
        A.atts_classify_ordinal(calib, test[i % len(test)], list(wl.alphas), None, None, cls, None)
    torch.cuda.synchronize()
    dt_cls = A.atts_profile_read(A.STAGES.index("classify"))[0] / steps * 1e-3
    A.atts_profile_enable(False)
    n_mid2 = n_mid + n_new * steps
    # bytes the method must move per step: read the set once, read + append the new scores, read the test
    # scores, write ranks (4 B) and classes (1 B).  Keeping the set sorted adds one more pass: the merge reads
    # the old array and writes the new one.
    bytes_step = 4 * n_mid + 8 * n_new + 4 * n_test + 5 * n_test
    merge_bytes = 4 * n_mid2 + 4 * n_new + 4 * (n_mid2 + n_new) * (1 + 1 / 32 + 1 / 1024)   # old + batch in, array + index out
    out = {
        "workload": (f"calib{' (scaled, out of cache)' if scaled else ''}: {n_cal} lognormal scores + {n_new} appended and "
                     f"{n_test} classified per step, alphas {list(wl.alphas)}"),
        "steps": steps, "us_per_step": dt / steps * 1e6, "decisions_per_s": n_test * steps / dt,
        "algorithmic_bytes_per_step": bytes_step, "achieved_GBs": bytes_step * steps / dt / 1e9,
        "hbm_frac": bytes_step * steps / dt / 1e9 / HBM_PEAK_GBS,
        "stage_us": st,
        "classes_only": {"device_us_per_call": dt_cls * 1e6, "decisions_per_s": n_test / dt_cls,
                         "achieved_GBs": 5 * n_test / dt_cls / 1e9, "hbm_frac": 5 * n_test / dt_cls / 1e9 / HBM_PEAK_GBS},
        "merge_kernel": {"bytes_per_launch": merge_bytes, "avg_launch_us": st["calib_merge"],
                         "achieved_GBs": merge_bytes / (st["calib_merge"] * 1e-6) / 1e9 if st["calib_merge"] > 0 else 0.0,
                         "hbm_frac": merge_bytes / (st["calib_merge"] * 1e-6) / 1e9 / HBM_PEAK_GBS if st["calib_merge"] > 0 else 0.0},
    }
    if not scaled:
        out["note"] = "working set (4-8 MB) is cache resident and a step is a few short kernels: latency bound, not HBM bound"
    if cpu:
        host_draw = lambda n, seed: lognormal_scores(n, wl.seed + 5000 + seed)
        if scaled:       # a bounded sample: 1/16 of the resident set and of the batches
            out["cpu_baseline"] = calibration_cpu_baseline(
                np, torch, n_cal >> 4, n_new >> 4, n_test >> 4, list(wl.alphas), host_draw, 2,
                f"numpy fp64 oracle (sort + binary search), 2 steps at 1/16 of the sizes: {n_cal >> 4} resident scores, "
                f"{n_new >> 4} appended and {n_test >> 4} classified per step")
        else:
            out["cpu_baseline"] = calibration_cpu_baseline(
                np, torch, n_cal, n_new, n_test, list(wl.alphas), host_draw, 4,
                f"numpy fp64 oracle (sort + binary search), 4 full steps of the workload: {n_cal} resident scores, {n_new} appended "
                f"and {n_test} classified per step")
    return out


def bench_conditional(A, torch, np, S=4096, m=64, k=64, reps=20):
    """Conditional coverage: S inputs, each ranks its k candidates against its own m calibration scores."""
    from synth import WORKLOADS, lognormal_scores
    wl = WORKLOADS["calib"]
    cal = torch.from_numpy(lognormal_scores(S * m, wl.seed + 31)).cuda()
    test = torch.from_numpy(lognormal_scores(S * k, wl.seed + 32)).cuda()
    cal_off = torch.arange(0, S * m + 1, m, dtype=torch.int64, device="cuda")
    test_off = torch.arange(0, S * k + 1, k, dtype=torch.int64, device="cuda")
    ranks = torch.empty(S * k, dtype=torch.int32, device="cuda")
    cls = torch.empty(S * k, dtype=torch.uint8, device="cuda")
    for _ in range(3):
        A.atts_classify_conditional(cal, cal_off, test, test_off, list(wl.alphas), ranks, None, cls)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        A.atts_classify_conditional(cal, cal_off, test, test_off, list(wl.alphas), ranks, None, cls)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps
    return {"workload": f"{S} inputs x {m} own calibration scores x {k} candidates, alphas {list(wl.alphas)}",
            "us_per_call": dt * 1e6, "decisions_per_s": S * k / dt, "comparisons_per_s": S * m * k / dt}


def bench_decision_flips(A, torch, np, n_batches=25):
    """End-to-end decision flips: config 1 (Tiny: 200 calibration scores from 25 batches of 8 drafts, alpha 0.1), the same
    token ids through the HIP path and through the oracle; every candidate of 25 further batches is classified by the
    same rule on each side with that side's own scores.  A flip = a candidate whose two classes differ; it can only come
    from the score error (the classifiers agree bit for bit given equal scores).  Done for the fp32 model and for the
    same architecture stored in bf16."""
    import dataclasses
    from oracle import atts_oracle as O
    from synth import WORKLOADS, make_token_ids, make_weights
    wl = WORKLOADS["tiny"]
    res = {}
    for dtype in ("fp32", "bf16"):
        cfg = dataclasses.replace(wl.model, dtype=dtype)
        w = make_weights(cfg, wl.seed, device="cuda")
        w_np = {k: ([t.float().cpu().numpy() for t in v] if isinstance(v, list) else v.float().cpu().numpy()) for k, v in w.items()}
        model = A.Model(cfg, w)
        ws = torch.empty(A.atts_workspace_bytes(model, wl.P, wl.K, wl.T), dtype=torch.uint8, device="cuda")
        sc = torch.empty(wl.K, dtype=torch.float32, device="cuda")
        g_scores, o_scores = [], []
        for i in range(2 * n_batches):
            pi, di = make_token_ids(cfg.vocab, wl.P, wl.K, wl.T, wl.seed + 300007 + i, device="cuda")
            A.atts_score_drafts(model, pi, di, None, A.SCORE_MEAN_NLL, None, sc, ws)
            g_scores.append(sc.cpu().numpy().copy())
            o_scores.append(O.score_drafts(w_np, cfg, pi.cpu().numpy(), di.cpu().numpy())[1].astype(np.float32))
        g = np.concatenate(g_scores)
        o = np.concatenate(o_scores)
        n_cal = n_batches * wl.K
        calib = A.Calib(n_cal)
        A.atts_calibrate_online(calib, torch.from_numpy(g[:n_cal]).cuda())
        test = torch.from_numpy(g[n_cal:]).cuda()
        ranks = torch.empty(test.numel(), dtype=torch.int32, device="cuda")
        cls = torch.empty(test.numel(), dtype=torch.uint8, device="cuda")
        A.atts_classify_ordinal(calib, test, list(wl.alphas), ranks, None, cls, None)
        torch.cuda.synchronize()
        oc = O.CalibrationSet()
        oc.append(o[:n_cal])
        o_cls = oc.classify(o[n_cal:], list(wl.alphas))[2]
        g_cls = cls.cpu().numpy()
        res[dtype] = {"candidates": int(test.numel()), "n_cal": n_cal, "flips": int((g_cls != o_cls).sum()),
                      "rejected_gpu": int((g_cls > 0).sum()), "rejected_oracle": int((o_cls > 0).sum()),
                      "max_abs_score_error": float(np.abs(g.astype(np.float64) - o).max()),
                      "score_std": float(o.std())}
        calib.close()
    return {"workload": f"tiny (config 1): {n_batches} calibration + {n_batches} test batches of K={wl.K} x T={wl.T}, alpha={list(wl.alphas)}",
            **res}


def bench_sync_vs_async(A, torch, np, model, cfg, wl, cal_scores, t_m_ms, requests=(2, 4, 8), n_streams=2):
    """Asynchronous arithmetic intensity r = T_c / (T_m + T_s) (Sec. "Q1") of both designs with several requests in
    flight.  A turn = R requests (inputs), each scoring its m = K candidates with one atts_score_drafts call, the calls
    spread over `n_streams` HIP streams.
      asynchronous (the method): a request's candidates are ranked against the calibration set as soon as its own
        scores exist (atts_classify_ordinal on the request's stream); T_s = that launch.
      synchronous (classic setup): normalise over each input's m candidates, global threshold over ALL normalised
        calibration + turn scores (a sort), prediction sets; the chain starts when the LAST request of the turn has
        been scored, so T_s of a request = wait for the others + the chain.
    T_c = scoring time per request (wall time of the turn's scoring / R); T_m = the memory-bound stages of one scoring
    pass (from the stage timers of the headline step)."""
    m = wl.K
    streams = [torch.cuda.Stream() for _ in range(n_streams)]
    ws = [torch.empty(A.atts_workspace_bytes(model, wl.P, wl.K, wl.T), dtype=torch.uint8, device="cuda") for _ in range(n_streams)]
    r_max = max(requests)
    from synth import make_token_ids
    ids = [make_token_ids(cfg.vocab, wl.P, wl.K, wl.T, wl.seed + 1100001 + i, device="cuda") for i in range(r_max)]
    sc = torch.empty(r_max, m, dtype=torch.float32, device="cuda")
    ranks = torch.empty(r_max, m, dtype=torch.int32, device="cuda")
    cls = torch.empty(r_max, m, dtype=torch.uint8, device="cuda")
    n_cal_in = cal_scores.numel() // m
    cal_nll = cal_scores[: n_cal_in * m].view(n_cal_in, m).contiguous()
    calib = A.Calib(cal_nll.numel() + 16 * r_max * m)
    A.atts_calibrate_online(calib, cal_nll.view(-1))
    cap = cal_nll.numel() + r_max * m
    s_all = torch.empty(cap, dtype=torch.float32, device="cuda")                    # normalised calibration scores, then the turn's
    A.atts_classic_normalize(cal_nll, s_all[: cal_nll.numel()].view(n_cal_in, m))
    tau = torch.empty(1, dtype=torch.float32, device="cuda")
    member = torch.empty(r_max, m, dtype=torch.uint8, device="cuda")
    cws = torch.empty(A.atts_classic_workspace_bytes(cap), dtype=torch.uint8, device="cuda")
    main = torch.cuda.current_stream()
    ev = lambda: torch.cuda.Event(enable_timing=True)
    out = {}
    for R in requests:
        res = {}
        for design in ("asynchronous", "synchronous"):
            for rep in range(2):                                                    # the first repetition warms up
                start, scored, decided = ev(), [ev() for _ in range(R)], [ev() for _ in range(R)]
                torch.cuda.synchronize()
                start.record(main)
                for st in streams:
                    st.wait_event(start)
                for r in range(R):
                    st = streams[r % n_streams]
                    with torch.cuda.stream(st):
                        p, d = ids[r]
                        A.atts_score_drafts(model, p, d, None, A.SCORE_MEAN_NLL, None, sc[r], ws[r % n_streams])
                        scored[r].record(st)
                        if design == "asynchronous":
                            A.atts_classify_ordinal(calib, sc[r], list(wl.alphas), ranks[r], None, cls[r], None)
                            decided[r].record(st)
                for r in range(R):
                    main.wait_event(scored[r])
                if design == "synchronous":
                    n0 = cal_nll.numel()
                    A.atts_classic_normalize(sc[:R], s_all[n0: n0 + R * m].view(R, m))
                    A.atts_classic_threshold(s_all[: n0 + R * m], wl.alphas[-1], tau, cws)
                    A.atts_classic_prediction_sets(s_all[n0: n0 + R * m], tau, member[:R].view(-1))
                    end = ev()
                    end.record(main)
                    decided = [end] * R
                torch.cuda.synchronize()
            t_scoring = max(start.elapsed_time(e) for e in scored)
            t_s = [scored[r].elapsed_time(decided[r]) for r in range(R)]
            t_c = t_scoring / R
            res[design] = {"T_c_ms": t_c, "T_s_ms_mean": float(np.mean(t_s)), "T_s_ms_max": float(np.max(t_s)),
                           "r": t_c / (t_m_ms + float(np.mean(t_s)))}
        out[f"R={R}"] = res
    calib.close()
    return {"workload": (f"{wl.name}: turns of R requests x m={m} candidates x T={wl.T} tokens, prefix {wl.P}, {n_streams} streams; "
                         f"{cal_nll.numel()} calibration scores; T_m = {t_m_ms:.3f} ms per request"),
            "definition": "r = T_c / (T_m + T_s); T_s = time from a request's scores being ready to its decisions being ready",
            **out}


def bench_warm_prefix(A, torch, model, cfg, wl, L, steps=5):
    """The headline workload with its prefix prefilled once (atts_prefix_extend) and kept in a handle: a step scores
    the K drafts against the cached prefix keys / values (only the K T draft rows go through the model)."""
    from synth import make_token_ids
    pre = A.Prefix(model, wl.P)
    p, _ = make_token_ids(cfg.vocab, wl.P, wl.K, wl.T, wl.seed + 500001, device="cuda")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    A.atts_prefix_extend(pre, p, torch.empty(A.atts_prefix_extend_workspace_bytes(pre, wl.P), dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    t_prefill = time.perf_counter() - t0
    ws = torch.empty(A.atts_workspace_bytes(model, wl.P, wl.K, wl.T), dtype=torch.uint8, device="cuda")
    sc = torch.empty(wl.K, dtype=torch.float32, device="cuda")
    drafts = [make_token_ids(cfg.vocab, wl.P, wl.K, wl.T, wl.seed + 500002 + i, device="cuda")[1] for i in range(steps + 1)]
    A.atts_score_drafts_cached(pre, drafts[0], None, A.SCORE_MEAN_NLL, None, sc, ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(1, steps + 1):
        A.atts_score_drafts_cached(pre, drafts[i], None, A.SCORE_MEAN_NLL, None, sc, ws)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    fl = algorithmic_flops(cfg, wl.P, wl.K, wl.T, L)
    fl0 = algorithmic_flops(cfg, wl.P, 0, 1, L)                 # the prefix rows alone (no LM head)
    warm = fl["total"] - (fl0["total"] - fl0["lmhead"])
    return {"workload": f"{wl.name}: prefix of {wl.P} tokens cached, K={wl.K} x T={wl.T} scored per step", "steps": steps,
            "prefill_ms": t_prefill * 1e3, "ms_per_step": dt * 1e3, "scored_tokens_per_s": wl.K * wl.T / dt,
            "algorithmic_tflop_per_step": warm / 1e12,
            "mfma_frac": warm / dt / 1e12 / MFMA_PEAK_TFLOPS[cfg.dtype]}


def bench_continuation(A, torch, model, cfg, wl, L, K=4, n_new=16):
    """Target-model continuation of K rejected candidates (about alpha K of a turn): prefix cached, each candidate's
    T-token draft as its own context, n_new greedy tokens each: one K-row pass per generated token."""
    from synth import make_token_ids
    pre = A.Prefix(model, wl.P)
    p, d = make_token_ids(cfg.vocab, wl.P, K, wl.T, wl.seed + 700001, device="cuda")
    A.atts_prefix_extend(pre, p, torch.empty(A.atts_prefix_extend_workspace_bytes(pre, wl.P), dtype=torch.uint8, device="cuda"))
    ws = torch.empty(A.atts_continue_workspace_bytes(pre, K, wl.T, n_new), dtype=torch.uint8, device="cuda")
    out = torch.empty(K, n_new, dtype=torch.int32, device="cuda")
    out1 = torch.empty(K, 1, dtype=torch.int32, device="cuda")
    def timed(o):
        A.atts_continue_greedy(pre, d, o, ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        A.atts_continue_greedy(pre, d, o, ws)
        torch.cuda.synchronize()
        return time.perf_counter() - t0
    t_full, t_one = timed(out), timed(out1)
    per_tok = (t_full - t_one) / (n_new - 1)            # the context pass + first token is common to both
    u = torch.rand(K, n_new, device="cuda", generator=torch.Generator(device="cuda").manual_seed(wl.seed))
    def timed_sampled(o, uu):
        A.atts_continue_sample(pre, d, 1.0, uu, o, ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        A.atts_continue_sample(pre, d, 1.0, uu, o, ws)
        torch.cuda.synchronize()
        return time.perf_counter() - t0
    per_tok_sampled = (timed_sampled(out, u) - timed_sampled(out1, u[:, :1].contiguous())) / (n_new - 1)
    esz = 2 if cfg.dtype == "bf16" else 4
    d_, hd = cfg.d_model, cfg.head_dim
    per_layer = d_ * (cfg.n_q_heads + 2 * cfg.n_kv_heads) * hd + cfg.n_q_heads * hd * d_ + 3 * d_ * cfg.d_ffn
    wbytes = esz * (per_layer * L + cfg.vocab * d_)
    return {"workload": f"{wl.name} model, prefix of {wl.P} cached, {K} candidates x {wl.T}-token drafts continued by {n_new} tokens",
            "context_pass_ms": t_one * 1e3, "ms_per_decode_step": per_tok * 1e3, "generated_tokens_per_s": K / per_tok,
            "ms_per_decode_step_sampled": per_tok_sampled * 1e3,
            "weight_bytes_per_step": wbytes, "achieved_GBs": wbytes / per_tok / 1e9, "hbm_frac": wbytes / per_tok / 1e9 / HBM_PEAK_GBS}


def bench_decode_shaped(A, torch, model, cfg, wl, L, K=16, T=8, steps=5):
    """The same resident model at a decode-like shape: the workload's prefix is cached in a prefix handle and only
    K T = 128 draft rows go through the model, well under the ~315 flop/byte ridge: one scoring pass must stream
    every layer's weights and the LM head from HBM once, so it is timed against the HBM roofline instead of the
    MFMA one."""
    from synth import make_token_ids
    pre = A.Prefix(model, wl.P)
    p, _ = make_token_ids(cfg.vocab, wl.P, K, T, wl.seed + 900000, device="cuda")
    A.atts_prefix_extend(pre, p, torch.empty(A.atts_prefix_extend_workspace_bytes(pre, wl.P), dtype=torch.uint8, device="cuda"))
    ws = torch.empty(A.atts_workspace_bytes(model, wl.P, K, T), dtype=torch.uint8, device="cuda")
    sc = torch.empty(K, dtype=torch.float32, device="cuda")
    ids = [make_token_ids(cfg.vocab, wl.P, K, T, wl.seed + 900001 + i, device="cuda")[1] for i in range(steps + 1)]
    A.atts_score_drafts_cached(pre, ids[0], None, A.SCORE_MEAN_NLL, None, sc, ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(1, steps + 1):
        A.atts_score_drafts_cached(pre, ids[i], None, A.SCORE_MEAN_NLL, None, sc, ws)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    esz = 2 if cfg.dtype == "bf16" else 4
    d, hd = cfg.d_model, cfg.head_dim
    per_layer = d * (cfg.n_q_heads + 2 * cfg.n_kv_heads) * hd + cfg.n_q_heads * hd * d + 3 * d * cfg.d_ffn
    wbytes = esz * (per_layer * L + cfg.vocab * d)
    return {"workload": f"{wl.name} model, prefix of {wl.P} tokens cached, K={K} T={T} ({K * T} rows through the model)",
            "steps": steps, "ms_per_pass": dt * 1e3, "scored_tokens_per_s": K * T / dt,
            "weight_bytes_per_pass": wbytes, "achieved_GBs": wbytes / dt / 1e9,
            "hbm_frac": wbytes / dt / 1e9 / HBM_PEAK_GBS}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="7b", choices=["tiny", "7b", "32b", "70b"])
    ap.add_argument("--layers", type=int, default=0, help="build only the first L layers (debug; result is labelled)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-layers", type=int, default=0,
                    help="layers of the model the CPU baseline times (0 = all of them; fewer are extrapolated to all by count and labelled)")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (reference for scaling HBM counters)")
    ap.add_argument("--skip-extras", action="store_true",
                    help="leave out the calibration-only, out-of-cache and decode-shaped measurements (profiling runs)")
    ap.add_argument("--legs", default="all",
                    help="comma-separated extra legs to run after the headline measurement: calib, calib_scaled, warm_prefix, "
                         "decode_shaped, conditional, continuation, sync_vs_async (default: all of them)")
    ap.add_argument("--calib-batches", type=int, default=-1,
                    help="scoring passes used to pre-sample the calibration set (-1: all ceil(n_cal / K) for tiny/7b, "
                         "2 for the larger models); the rest is drawn from a normal fitted to those scores")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures ONE MI355X; the path has no multi-GPU leg (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2509_15148_amd as A
    from synth import WORKLOADS, make_token_ids, make_weights

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    wl = WORKLOADS[args.workload]
    cfg = wl.model
    L = args.layers if args.layers > 0 else cfg.n_layers

    t0 = time.perf_counter()
    w = make_weights(cfg, wl.seed, device="cuda", n_layers=L)
    torch.cuda.synchronize()
    log(f"[bench] weights for {wl.name} ({L} layers) built in {time.perf_counter() - t0:.1f} s")
    model = A.Model(cfg, w)
    ws = torch.empty(A.atts_workspace_bytes(model, wl.P, wl.K, wl.T), dtype=torch.uint8, device="cuda")
    n_batches = args.warmup + args.steps
    n_cal_batches = math.ceil(wl.n_cal / wl.K)
    ids = [make_token_ids(cfg.vocab, wl.P, wl.K, wl.T, wl.seed + 17 * i, device="cuda")
           for i in range(max(n_batches, 1))]
    lp = torch.empty(wl.K, wl.T, dtype=torch.float32, device="cuda")
    sc = torch.empty(wl.K, dtype=torch.float32, device="cuda")
    ranks = torch.empty(wl.K, dtype=torch.int32, device="cuda")
    pv = torch.empty(wl.K, dtype=torch.float32, device="cuda")
    cls = torch.empty(wl.K, dtype=torch.uint8, device="cuda")
    thr = torch.empty(len(wl.alphas), dtype=torch.float32, device="cuda")

    # Pre-sampling pass of online calibration: n_cal scores from ceil(n_cal / K) extra batches
    # through the same scoring path (untimed set-up).
    calib = A.Calib(n_cal_batches * wl.K + (n_batches + args.steps) * wl.K)   # timed pass + stage-timing pass
    t0 = time.perf_counter()
    n_real = args.calib_batches if args.calib_batches >= 0 else (n_cal_batches if args.workload in ("tiny", "7b") else 2)
    n_real = max(1, min(n_real, n_cal_batches))
    seen = []
    for i in range(n_real):
        p, d = make_token_ids(cfg.vocab, wl.P, wl.K, wl.T, wl.seed + 100003 + i, device="cuda")
        A.atts_score_drafts(model, p, d, None, A.SCORE_MEAN_NLL, None, sc, ws)
        A.atts_calibrate_online(calib, sc)
        seen.append(sc.clone())
    seen = torch.cat(seen)
    if n_real < n_cal_batches:
        g = torch.Generator(device="cuda").manual_seed(wl.seed)
        fill = seen.mean() + seen.std() * torch.randn((n_cal_batches - n_real) * wl.K, device="cuda", generator=g)
        A.atts_calibrate_online(calib, fill.float().contiguous())
        seen = torch.cat([seen, fill.float()])
    torch.cuda.synchronize()
    calib_note = (f"{n_real} scoring passes" if n_real == n_cal_batches else
                  f"{n_real} scoring passes + {(n_cal_batches - n_real) * wl.K} scores from a normal fitted to them")
    log(f"[bench] calibration pre-sampling: {calib_note} in {time.perf_counter() - t0:.1f} s, "
        f"N = {A.atts_calib_size(calib)}")

    def step(i):
        p, d = ids[i % len(ids)]
        A.atts_score_drafts(model, p, d, None, A.SCORE_MEAN_NLL, lp, sc, ws)
        A.atts_classify_ordinal(calib, sc, list(wl.alphas), ranks, pv, cls, thr)
        A.atts_calibrate_online(calib, sc)

    if args.traffic_probe:
        src_buf = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst_buf = torch.empty_like(src_buf)
        dst_buf.copy_(src_buf)                     # 1 GiB read + 1 GiB written
        torch.cuda.synchronize()
        del src_buf, dst_buf

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_step = dt / args.steps * 1e3
    assert A.atts_model_check(model) == 0
    rej = float((cls > 0).float().mean())
    log(f"[bench] {args.steps} steps: {ms_step:.2f} ms/step; last batch scores {sc[:4].tolist()} reject frac {rej:.2f}")

    # Same steps again with per-stage HIP events on the launch stream (kernel-level durations).
    A.atts_profile_enable(True)
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    stage_ms = {}
    for s, name in enumerate(A.STAGES):
        ms, n = A.atts_profile_read(s)
        stage_ms[name] = (ms, n)
    A.atts_profile_enable(False)

    fl = algorithmic_flops(cfg, wl.P, wl.K, wl.T, L)
    peak = MFMA_PEAK_TFLOPS[cfg.dtype]
    stages = {}
    for name, (ms, n) in stage_ms.items():
        e = {"ms_per_step": ms / args.steps, "launches_per_step": n / args.steps}
        if name in fl and ms > 0:
            e["tflops"] = fl[name] * args.steps / (ms * 1e-3) / 1e12
            e["mfma_frac"] = e["tflops"] / peak
        stages[name] = e
    dom = "gemm_gate_up"
    dom_ms, dom_n = stage_ms[dom]
    dom_avg_ms = dom_ms / max(dom_n, 1)
    dom_flops = fl[dom] / max(L, 1)                      # one launch = one layer's gate/up projection
    achieved = dom_flops / (dom_avg_ms * 1e-3) / 1e12 if dom_avg_ms > 0 else 0.0

    # asynchronous arithmetic intensity r = T_c / (T_m + T_s) (Sec. "Q1"), from the per-stage device times of one step:
    # T_c = contraction stages (GEMMs, attention), T_m = the memory-bound stages between them, T_s = what the
    # conformal layer costs per step (rank / classify + online calibration; the synchronisation term of the
    # normalised-score design it replaces)
    t_c = sum(stages[k]["ms_per_step"] for k in ("gemm_qkv", "attention", "gemm_o", "gemm_gate_up", "gemm_down", "lmhead"))
    t_m = sum(stages[k]["ms_per_step"] for k in ("embed", "norm", "rope", "gather_norm", "reduce"))
    t_s = sum(stages[k]["ms_per_step"] for k in ("calib_sort", "calib_merge", "classify"))
    # the five GEMM stages taken together: their algorithmic flops over the sum of their device times
    gemm_names = ("gemm_qkv", "gemm_o", "gemm_gate_up", "gemm_down", "lmhead")
    gemm_ms = sum(stage_ms[k][0] for k in gemm_names)
    gemm_frac = (sum(fl[k] for k in gemm_names) * args.steps / (gemm_ms * 1e-3) / 1e12 / peak) if gemm_ms > 0 else None
    out = {
        "metric": "scored draft tokens/sec (shared-prefix target scoring + online conformal calibration + ordinal "
                  "classification), 1 MI355X",
        "value": wl.K * wl.T * args.steps / dt,
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: L={L} d={cfg.d_model} {cfg.n_q_heads}q/{cfg.n_kv_heads}kv x{cfg.head_dim} "
                               f"F={cfg.d_ffn} V={cfg.vocab} {cfg.dtype}; P={wl.P} K={wl.K} T={wl.T}; "
                               f"n_cal={A.atts_calib_size(calib)} alpha={list(wl.alphas)}",
                   "scored_tokens_per_step": wl.K * wl.T, "rows_per_step": wl.P + wl.K * wl.T,
                   "layers_built": L, "full_model": L == cfg.n_layers, "calibration_set": calib_note},
        "conformal_decisions_per_s": wl.K * args.steps / dt,
        "algorithmic_tflop_per_step": fl["total"] / 1e12,
        "whole_step_mfma_frac": fl["total"] / (dt / args.steps) / 1e12 / peak,
        "scoring_gemms_mfma_frac": gemm_frac,
        "roofline": {"bound": "mfma", "kernel": f"aligned {cfg.dtype} GEMM, SwiGLU epilogue (gate/up projection)",
                     "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                     "avg_launch_ms": dom_avg_ms, "flops_per_launch": dom_flops,
                     "traffic": measured_traffic(args.workload),
                     "traffic_source": "recorded constant from profiles/traffic_gemm_gate_up_7b.txt (rocprofv3 --pmc FETCH_SIZE / "
                                       "WRITE_SIZE), not measured by this run; null when csrc/gemm.hip has changed since"},
        "stages": stages,
        "async_arithmetic_intensity": {"T_c_ms": t_c, "T_m_ms": t_m, "T_s_ms": t_s, "r": t_c / (t_m + t_s) if t_m + t_s > 0 else None},
    }
    if args.workload != "tiny" and not args.skip_extras:
        legs = {"calib", "calib_scaled", "warm_prefix", "decode_shaped", "conditional", "continuation", "sync_vs_async"}
        if args.legs != "all":
            want = set(x for x in args.legs.split(",") if x)
            if not want <= legs:
                print(f"bench.py: unknown leg(s) {sorted(want - legs)}; known: {sorted(legs)}", file=sys.stderr)
                sys.exit(2)
            legs = want
        if "calib" in legs:
            out["calibration_stage"] = bench_calibration(A, torch, np, cpu=not args.no_cpu_baseline)
        if "calib_scaled" in legs:
            out["calibration_stage_scaled"] = bench_calibration(A, torch, np, steps=4, scaled=True, cpu=not args.no_cpu_baseline)
        if "warm_prefix" in legs:
            out["warm_prefix"] = bench_warm_prefix(A, torch, model, cfg, wl, L)
        if "decode_shaped" in legs:
            out["decode_shaped"] = bench_decode_shaped(A, torch, model, cfg, wl, L)
        if "conditional" in legs:
            out["conditional_stage"] = bench_conditional(A, torch, np)
        if "continuation" in legs:
            out["continuation"] = bench_continuation(A, torch, model, cfg, wl, L)
        if "sync_vs_async" in legs:
            out["sync_vs_async"] = bench_sync_vs_async(A, torch, np, model, cfg, wl, seen, t_m)
    if not args.no_cpu_baseline:
        p0, d0 = ids[0]
        out["decision_flips"] = bench_decision_flips(A, torch, np)
        out["cpu_baseline"] = cpu_baseline(cfg, wl, w, p0.cpu().numpy(), d0.cpu().numpy(), L,
                                           min(args.cpu_layers, L) if args.cpu_layers > 0 else L)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
