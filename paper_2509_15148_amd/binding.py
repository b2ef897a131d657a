"""ctypes binding of libatts.so: argument marshalling only.

Every function here has the name of the C entry point it calls (include/atts.h) and does
nothing but convert torch tensors to device pointers, check dtypes/contiguity, pick the
current HIP stream and raise AttsError on a non-zero status.  All arithmetic of the
method runs in the HIP kernels.  There is no CPU fallback: importing this module without a
built library raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libatts.so")

OK = 0
ERR_INVALID_ARG, ERR_SHAPE, ERR_WORKSPACE, ERR_CAPACITY, ERR_HIP = -1, -2, -3, -4, -5
DTYPE_F32, DTYPE_BF16 = 0, 1
SCORE_MEAN_NLL, SCORE_SUM_NLL = 0, 1
MAX_ALPHAS = 8

EXPORTS = (
    "atts_last_error_string", "atts_model_create", "atts_model_destroy", "atts_workspace_bytes",
    "atts_score_drafts", "atts_model_check", "atts_prefix_create", "atts_prefix_destroy", "atts_prefix_length",
    "atts_prefix_reset", "atts_prefix_extend_workspace_bytes", "atts_prefix_extend", "atts_score_drafts_cached",
    "atts_continue_workspace_bytes", "atts_continue_greedy", "atts_continue_sample", "atts_lmhead_workspace_bytes", "atts_lmhead_logprobs",
    "atts_lmhead_logprobs_static",
    "atts_gemm_nt", "atts_attention_workspace_bytes", "atts_attention_shared_prefix",
    "atts_calib_create", "atts_calib_destroy", "atts_calib_size", "atts_calib_reset",
    "atts_calibrate_online", "atts_classify_ordinal", "atts_classify_conditional", "atts_calib_export",
    "atts_calib_import", "atts_classic_workspace_bytes", "atts_classic_normalize", "atts_classic_threshold",
    "atts_classic_prediction_sets",
    "atts_profile_enable", "atts_profile_read",
)

STAGES = ("embed", "norm", "gemm_qkv", "rope", "attention", "gemm_o", "gemm_gate_up", "gemm_down", "gather_norm",
          "lmhead", "reduce", "calib_sort", "calib_merge", "classify")


class AttsError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"atts status {code}: {message}")
        self.code = code


class _ModelDesc(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("d_model", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("d_ffn", ctypes.c_int32),
                ("vocab", ctypes.c_int32), ("dtype", ctypes.c_int32), ("rope_theta", ctypes.c_float),
                ("rms_eps", ctypes.c_float)]


class _Weights(ctypes.Structure):
    _fields_ = [("tok_embed", ctypes.c_void_p), ("final_norm", ctypes.c_void_p), ("lm_head", ctypes.c_void_p),
                ("attn_norm", ctypes.POINTER(ctypes.c_void_p)), ("wqkv", ctypes.POINTER(ctypes.c_void_p)),
                ("wo", ctypes.POINTER(ctypes.c_void_p)), ("ffn_norm", ctypes.POINTER(ctypes.c_void_p)),
                ("w_gate_up", ctypes.POINTER(ctypes.c_void_p)), ("w_down", ctypes.POINTER(ctypes.c_void_p))]


def load_library(path: str = LIB_PATH) -> ctypes.CDLL:
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2509_15148_amd.build` "
                          "(there is no CPU fallback)")
    lib = ctypes.CDLL(path)
    lib.atts_last_error_string.restype = ctypes.c_char_p
    for name in EXPORTS:
        fn = getattr(lib, name)            # AttributeError if a declared symbol is not exported
        if name != "atts_last_error_string":
            fn.restype = ctypes.c_int32
    return lib


_lib = load_library()


def _check(rc: int) -> None:
    if rc != OK:
        raise AttsError(rc, _lib.atts_last_error_string().decode())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t: Optional[torch.Tensor], dtype=None, name="tensor") -> ctypes.c_void_p:
    if t is None:
        return ctypes.c_void_p(0)
    if not t.is_cuda:
        raise AttsError(ERR_INVALID_ARG, f"{name} must be a device tensor")
    if not t.is_contiguous():
        raise AttsError(ERR_INVALID_ARG, f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise AttsError(ERR_INVALID_ARG, f"{name} must have dtype {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _dtype_code(dt: torch.dtype) -> int:
    if dt == torch.float32:
        return DTYPE_F32
    if dt == torch.bfloat16:
        return DTYPE_BF16
    raise AttsError(ERR_INVALID_ARG, f"unsupported dtype {dt}")


class Model:
    """Handle from atts_model_create; keeps the weight tensors alive (they are borrowed)."""

    def __init__(self, cfg, weights: Dict[str, object]):
        L = len(weights["wqkv"])
        self.cfg = cfg
        self.n_layers = L
        self._keep = weights
        mat_dt = weights["lm_head"].dtype
        desc = _ModelDesc(L, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn, cfg.vocab,
                          _dtype_code(mat_dt), cfg.rope_theta, cfg.rms_eps)
        w = _Weights()
        w.tok_embed = _ptr(weights["tok_embed"], mat_dt, "tok_embed")
        w.final_norm = _ptr(weights["final_norm"], torch.float32, "final_norm")
        w.lm_head = _ptr(weights["lm_head"], mat_dt, "lm_head")
        self._arrays = []
        for key, dt in (("attn_norm", torch.float32), ("wqkv", mat_dt), ("wo", mat_dt), ("ffn_norm", torch.float32),
                        ("w_gate_up", mat_dt), ("w_down", mat_dt)):
            arr = (ctypes.c_void_p * max(L, 1))(*[_ptr(t, dt, f"{key}[{i}]") for i, t in enumerate(weights[key])])
            self._arrays.append(arr)
            setattr(w, key, ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p)))
        self.handle = ctypes.c_void_p()
        _check(_lib.atts_model_create(ctypes.byref(desc), ctypes.byref(w), ctypes.byref(self.handle)))

    def close(self) -> None:
        if self.handle:
            _lib.atts_model_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def atts_workspace_bytes(model: Model, P: int, K: int, T_max: int) -> int:
    out = ctypes.c_size_t()
    _check(_lib.atts_workspace_bytes(model.handle, P, K, T_max, ctypes.byref(out)))
    return out.value


def atts_score_drafts(model: Model, prefix_ids: torch.Tensor, draft_ids: torch.Tensor,
                      draft_lens: Optional[torch.Tensor], score_mode: int, token_logprobs: Optional[torch.Tensor],
                      scores: torch.Tensor, workspace: torch.Tensor) -> None:
    K, T_max = draft_ids.shape
    if token_logprobs is not None and tuple(token_logprobs.shape) != (K, T_max):
        raise AttsError(ERR_INVALID_ARG, "token_logprobs must be [K, T_max]")
    if scores.numel() != K or (draft_lens is not None and draft_lens.numel() != K):
        raise AttsError(ERR_INVALID_ARG, "scores / draft_lens must have K elements")
    _check(_lib.atts_score_drafts(
        model.handle, _ptr(prefix_ids, torch.int32, "prefix_ids"), ctypes.c_int32(prefix_ids.numel()),
        _ptr(draft_ids, torch.int32, "draft_ids"), _ptr(draft_lens, torch.int32, "draft_lens"),
        ctypes.c_int32(K), ctypes.c_int32(T_max), ctypes.c_int32(score_mode),
        _ptr(token_logprobs, torch.float32, "token_logprobs"), _ptr(scores, torch.float32, "scores"),
        _ptr(workspace, torch.uint8, "workspace"), ctypes.c_size_t(workspace.numel()), _stream()))


class Prefix:
    """Handle from atts_prefix_create (keys / values of a prompt prefix, kept across turns); keeps the model alive."""

    def __init__(self, model: Model, capacity: int):
        self.model = model
        self.handle = ctypes.c_void_p()
        _check(_lib.atts_prefix_create(model.handle, ctypes.c_int32(capacity), ctypes.byref(self.handle)))

    def close(self) -> None:
        if self.handle:
            _lib.atts_prefix_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def atts_prefix_length(prefix: Prefix) -> int:
    out = ctypes.c_int32()
    _check(_lib.atts_prefix_length(prefix.handle, ctypes.byref(out)))
    return out.value


def atts_prefix_reset(prefix: Prefix) -> None:
    _check(_lib.atts_prefix_reset(prefix.handle))


def atts_prefix_extend_workspace_bytes(prefix: Prefix, n: int) -> int:
    out = ctypes.c_size_t()
    _check(_lib.atts_prefix_extend_workspace_bytes(prefix.handle, ctypes.c_int32(n), ctypes.byref(out)))
    return out.value


def atts_prefix_extend(prefix: Prefix, ids: torch.Tensor, workspace: torch.Tensor) -> None:
    _check(_lib.atts_prefix_extend(prefix.handle, _ptr(ids, torch.int32, "ids"), ctypes.c_int32(ids.numel()),
                                   _ptr(workspace, torch.uint8, "workspace"), ctypes.c_size_t(workspace.numel()),
                                   _stream()))


def atts_score_drafts_cached(prefix: Prefix, draft_ids: torch.Tensor, draft_lens: Optional[torch.Tensor], score_mode: int,
                             token_logprobs: Optional[torch.Tensor], scores: torch.Tensor,
                             workspace: torch.Tensor) -> None:
    K, T_max = draft_ids.shape
    if token_logprobs is not None and tuple(token_logprobs.shape) != (K, T_max):
        raise AttsError(ERR_INVALID_ARG, "token_logprobs must be [K, T_max]")
    if scores.numel() != K or (draft_lens is not None and draft_lens.numel() != K):
        raise AttsError(ERR_INVALID_ARG, "scores / draft_lens must have K elements")
    _check(_lib.atts_score_drafts_cached(
        prefix.handle, _ptr(draft_ids, torch.int32, "draft_ids"), _ptr(draft_lens, torch.int32, "draft_lens"),
        ctypes.c_int32(K), ctypes.c_int32(T_max), ctypes.c_int32(score_mode),
        _ptr(token_logprobs, torch.float32, "token_logprobs"), _ptr(scores, torch.float32, "scores"),
        _ptr(workspace, torch.uint8, "workspace"), ctypes.c_size_t(workspace.numel()), _stream()))


def atts_continue_workspace_bytes(prefix: Prefix, K: int, T: int, n_new: int) -> int:
    out = ctypes.c_size_t()
    _check(_lib.atts_continue_workspace_bytes(prefix.handle, ctypes.c_int32(K), ctypes.c_int32(T), ctypes.c_int32(n_new),
                                              ctypes.byref(out)))
    return out.value


def atts_continue_greedy(prefix: Prefix, draft_ids: torch.Tensor, out_ids: torch.Tensor, workspace: torch.Tensor,
                         draft_lens: Optional[torch.Tensor] = None, eos_id: int = -1) -> None:
    K, T = draft_ids.shape
    if out_ids.dim() != 2 or out_ids.shape[0] != K or (draft_lens is not None and draft_lens.numel() != K):
        raise AttsError(ERR_INVALID_ARG, "out_ids must be [K, n_new], draft_lens [K]")
    _check(_lib.atts_continue_greedy(prefix.handle, _ptr(draft_ids, torch.int32, "draft_ids"), _ptr(draft_lens, torch.int32, "draft_lens"),
                                     ctypes.c_int32(K), ctypes.c_int32(T), ctypes.c_int32(out_ids.shape[1]), ctypes.c_int32(eos_id),
                                     _ptr(out_ids, torch.int32, "out_ids"), _ptr(workspace, torch.uint8, "workspace"),
                                     ctypes.c_size_t(workspace.numel()), _stream()))


def atts_continue_sample(prefix: Prefix, draft_ids: torch.Tensor, temperature: float, uniforms: torch.Tensor,
                         out_ids: torch.Tensor, workspace: torch.Tensor, draft_lens: Optional[torch.Tensor] = None,
                         eos_id: int = -1) -> None:
    K, T = draft_ids.shape
    if out_ids.dim() != 2 or out_ids.shape[0] != K or tuple(uniforms.shape) != tuple(out_ids.shape):
        raise AttsError(ERR_INVALID_ARG, "out_ids and uniforms must both be [K, n_new]")
    if draft_lens is not None and draft_lens.numel() != K:
        raise AttsError(ERR_INVALID_ARG, "draft_lens must have K elements")
    _check(_lib.atts_continue_sample(prefix.handle, _ptr(draft_ids, torch.int32, "draft_ids"), _ptr(draft_lens, torch.int32, "draft_lens"),
                                     ctypes.c_int32(K), ctypes.c_int32(T), ctypes.c_int32(out_ids.shape[1]), ctypes.c_int32(eos_id),
                                     ctypes.c_float(temperature), _ptr(uniforms, torch.float32, "uniforms"),
                                     _ptr(out_ids, torch.int32, "out_ids"), _ptr(workspace, torch.uint8, "workspace"),
                                     ctypes.c_size_t(workspace.numel()), _stream()))


def atts_model_check(model: Model) -> int:
    flag = ctypes.c_int32(-1)
    _check(_lib.atts_model_check(model.handle, _stream(), ctypes.byref(flag)))
    return flag.value


def atts_lmhead_workspace_bytes(B: int, V: int) -> int:
    out = ctypes.c_size_t()
    _check(_lib.atts_lmhead_workspace_bytes(B, V, ctypes.byref(out)))
    return out.value


def atts_lmhead_logprobs(x: torch.Tensor, w: torch.Tensor, targets: torch.Tensor, logprobs: torch.Tensor,
                         workspace: torch.Tensor) -> None:
    B, d = x.shape
    V = w.shape[0]
    if w.shape[1] != d or targets.numel() != B or logprobs.numel() != B:
        raise AttsError(ERR_INVALID_ARG, "shape mismatch")
    _check(_lib.atts_lmhead_logprobs(_dtype_code(x.dtype), _ptr(x, None, "x"), _ptr(w, x.dtype, "w"),
                                     _ptr(targets, torch.int32, "targets"), B, d, V,
                                     _ptr(logprobs, torch.float32, "logprobs"),
                                     _ptr(workspace, torch.uint8, "workspace"), ctypes.c_size_t(workspace.numel()),
                                     _stream()))


def atts_lmhead_logprobs_static(x: torch.Tensor, w: torch.Tensor, targets: torch.Tensor, logprobs: torch.Tensor) -> None:
    B, d = x.shape
    V = w.shape[0]
    if w.shape[1] != d or targets.numel() != B or logprobs.numel() != B:
        raise AttsError(ERR_INVALID_ARG, "shape mismatch")
    _check(_lib.atts_lmhead_logprobs_static(_dtype_code(x.dtype), _ptr(x, None, "x"), _ptr(w, x.dtype, "w"),
                                            _ptr(targets, torch.int32, "targets"), B, d, V,
                                            _ptr(logprobs, torch.float32, "logprobs"), _stream()))


def atts_gemm_nt(a: torch.Tensor, w: torch.Tensor, c: torch.Tensor) -> None:
    M, Kd = a.shape
    N = w.shape[0]
    if w.shape[1] != Kd or tuple(c.shape) != (M, N):
        raise AttsError(ERR_INVALID_ARG, "shape mismatch")
    _check(_lib.atts_gemm_nt(_dtype_code(a.dtype), _ptr(a, None, "a"), _ptr(w, a.dtype, "w"),
                             _ptr(c, torch.float32, "c"), M, N, Kd, _stream()))


def atts_attention_workspace_bytes(dtype: torch.dtype, R: int, n_kv: int, hd: int) -> int:
    out = ctypes.c_size_t()
    _check(_lib.atts_attention_workspace_bytes(_dtype_code(dtype), R, n_kv, hd, ctypes.byref(out)))
    return out.value


def atts_attention_shared_prefix(qkv: torch.Tensor, out: torch.Tensor, P: int, K: int, T: int, n_q: int, n_kv: int,
                                 hd: int, workspace: Optional[torch.Tensor]) -> None:
    R = P + K * T
    if tuple(qkv.shape) != (R, (n_q + 2 * n_kv) * hd) or tuple(out.shape) != (R, n_q * hd):
        raise AttsError(ERR_INVALID_ARG, "shape mismatch")
    _check(_lib.atts_attention_shared_prefix(
        _dtype_code(qkv.dtype), _ptr(qkv, None, "qkv"), _ptr(out, qkv.dtype, "out"), P, K, T, n_q, n_kv, hd,
        _ptr(workspace, torch.uint8, "workspace"),
        ctypes.c_size_t(0 if workspace is None else workspace.numel()), _stream()))


class Calib:
    """Handle from atts_calib_create."""

    def __init__(self, capacity: int):
        self.handle = ctypes.c_void_p()
        _check(_lib.atts_calib_create(ctypes.c_int64(capacity), ctypes.byref(self.handle)))

    def close(self) -> None:
        if self.handle:
            _lib.atts_calib_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def atts_calib_size(calib: Calib) -> int:
    n = ctypes.c_int64()
    _check(_lib.atts_calib_size(calib.handle, ctypes.byref(n)))
    return n.value


def atts_calib_reset(calib: Calib) -> None:
    _check(_lib.atts_calib_reset(calib.handle))


def atts_calibrate_online(calib: Calib, new_scores: torch.Tensor) -> None:
    _check(_lib.atts_calibrate_online(calib.handle, _ptr(new_scores, torch.float32, "new_scores"),
                                      ctypes.c_int64(new_scores.numel()), _stream()))


def atts_classify_ordinal(calib: Calib, test_scores: torch.Tensor, alphas: Sequence[float],
                          ranks: Optional[torch.Tensor], pvalues: Optional[torch.Tensor], classes: torch.Tensor,
                          thresholds: Optional[torch.Tensor]) -> None:
    M = test_scores.numel()
    if (ranks is not None and ranks.numel() != M) or classes.numel() != M or (pvalues is not None and pvalues.numel() != M):
        raise AttsError(ERR_INVALID_ARG, "ranks / pvalues / classes must have M elements")
    if thresholds is not None and thresholds.numel() != len(alphas):
        raise AttsError(ERR_INVALID_ARG, "thresholds must have n_alpha elements")
    arr = (ctypes.c_double * max(len(alphas), 1))(*[float(a) for a in alphas])
    _check(_lib.atts_classify_ordinal(calib.handle, _ptr(test_scores, torch.float32, "test_scores"),
                                      ctypes.c_int64(M), arr, ctypes.c_int32(len(alphas)),
                                      _ptr(ranks, torch.int32, "ranks"), _ptr(pvalues, torch.float32, "pvalues"),
                                      _ptr(classes, torch.uint8, "classes"),
                                      _ptr(thresholds, torch.float32, "thresholds"), _stream()))


def atts_classify_conditional(cal_scores: torch.Tensor, cal_offsets: torch.Tensor, test_scores: torch.Tensor,
                              test_offsets: torch.Tensor, alphas: Sequence[float], ranks: torch.Tensor,
                              pvalues: Optional[torch.Tensor], classes: torch.Tensor) -> None:
    n_inputs = cal_offsets.numel() - 1
    if n_inputs < 0 or test_offsets.numel() != n_inputs + 1:
        raise AttsError(ERR_INVALID_ARG, "cal_offsets and test_offsets must both have n_inputs + 1 elements")
    M = test_scores.numel()
    if ranks.numel() != M or classes.numel() != M or (pvalues is not None and pvalues.numel() != M):
        raise AttsError(ERR_INVALID_ARG, "ranks / pvalues / classes must have one element per test score")
    arr = (ctypes.c_double * max(len(alphas), 1))(*[float(a) for a in alphas])
    if n_inputs > 0:                       # the library wants non-NULL arrays; an empty tensor has no address
        spare = torch.zeros(1, dtype=torch.float32, device=cal_offsets.device)
        cal_scores = cal_scores if cal_scores.numel() else spare
        if M == 0:
            test_scores, ranks, classes = spare, spare.to(torch.int32), spare.to(torch.uint8)
            pvalues = None
    _check(_lib.atts_classify_conditional(_ptr(cal_scores, torch.float32, "cal_scores"),
                                          _ptr(cal_offsets, torch.int64, "cal_offsets"),
                                          _ptr(test_scores, torch.float32, "test_scores"),
                                          _ptr(test_offsets, torch.int64, "test_offsets"), ctypes.c_int64(n_inputs),
                                          arr, ctypes.c_int32(len(alphas)), _ptr(ranks, torch.int32, "ranks"),
                                          _ptr(pvalues, torch.float32, "pvalues"), _ptr(classes, torch.uint8, "classes"),
                                          _stream()))


def atts_calib_export(calib: Calib, out: torch.Tensor) -> None:
    _check(_lib.atts_calib_export(calib.handle, _ptr(out, torch.float32, "out"), _stream()))


def atts_calib_import(calib: Calib, scores: torch.Tensor) -> None:
    _check(_lib.atts_calib_import(calib.handle, _ptr(scores, torch.float32, "scores") if scores.numel() else ctypes.c_void_p(0),
                                  ctypes.c_int64(scores.numel()), _stream()))


def atts_classic_workspace_bytes(n_scores: int) -> int:
    out = ctypes.c_size_t()
    _check(_lib.atts_classic_workspace_bytes(ctypes.c_int64(n_scores), ctypes.byref(out)))
    return out.value


def atts_classic_normalize(nll: torch.Tensor, scores: torch.Tensor) -> None:
    if nll.dim() != 2 or tuple(scores.shape) != tuple(nll.shape):
        raise AttsError(ERR_INVALID_ARG, "nll and scores must both be [n_inputs, m]")
    _check(_lib.atts_classic_normalize(_ptr(nll, torch.float32, "nll"), ctypes.c_int64(nll.shape[0]), ctypes.c_int32(nll.shape[1]),
                                       _ptr(scores, torch.float32, "scores"), _stream()))


def atts_classic_threshold(cal_scores: torch.Tensor, alpha: float, tau: torch.Tensor, workspace: torch.Tensor) -> None:
    if tau.numel() != 1:
        raise AttsError(ERR_INVALID_ARG, "tau must have one element")
    _check(_lib.atts_classic_threshold(_ptr(cal_scores, torch.float32, "cal_scores"), ctypes.c_int64(cal_scores.numel()),
                                       ctypes.c_double(alpha), _ptr(tau, torch.float32, "tau"),
                                       _ptr(workspace, torch.uint8, "workspace"), ctypes.c_size_t(workspace.numel()), _stream()))


def atts_classic_prediction_sets(scores: torch.Tensor, tau: torch.Tensor, member: torch.Tensor) -> None:
    if member.numel() != scores.numel() or tau.numel() != 1:
        raise AttsError(ERR_INVALID_ARG, "member must have one element per score, tau one element")
    _check(_lib.atts_classic_prediction_sets(_ptr(scores, torch.float32, "scores"), ctypes.c_int64(scores.numel()),
                                             _ptr(tau, torch.float32, "tau"), _ptr(member, torch.uint8, "member"), _stream()))


def atts_profile_enable(on: bool) -> None:
    _check(_lib.atts_profile_enable(ctypes.c_int32(1 if on else 0)))


def atts_profile_read(stage: int):
    """-> (total device milliseconds, launches) of one stage since atts_profile_enable(True)."""
    ms, n = ctypes.c_double(), ctypes.c_int64()
    _check(_lib.atts_profile_read(ctypes.c_int32(stage), ctypes.byref(ms), ctypes.byref(n)))
    return ms.value, n.value
