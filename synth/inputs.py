"""Seeded synthetic workloads: model shapes, random-init weights, token ids, score samples.

Everything here is input generation.  The weight generator is a counter-based hash
(splitmix64 finaliser applied to ``element index + per-tensor base``) written with torch
integer ops only, so the same call produces bit-identical tensors on the CPU and on a
GPU: the oracle's tests can build weights on the host while a large benchmark builds
them directly in device memory.

Value recipe (random-init stand-in for trained checkpoints):
  * matrices:  uniform(-a, a), a = sqrt(3 / fan_in)  (std 1/sqrt(fan_in));
               the two residual-branch output projections (w_o, w_down) are further
               scaled by 1/sqrt(2 L) so the residual stream stays O(1) through L layers
  * embedding: uniform(-sqrt(3), sqrt(3))  (std 1)
  * norm gains: 1 + 0.1 * uniform(-1, 1)   (not exactly 1, so a dropped gain is visible)
  * stored dtype: fp32, or bf16 by round-to-nearest-even of the fp32 value
  * token ids:  uniform over [0, vocab)
  * conformal scores for the calibration-only workload: lognormal(0, 1), drawn in
    fp64 and rounded once to fp32
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional

import numpy as np
import torch

_MASK64 = (1 << 64) - 1


def _s64(x: int) -> int:
    """Reinterpret an unsigned 64-bit python int as signed (torch has no uint64 math)."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


def _mix64_int(x: int) -> int:
    x &= _MASK64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _MASK64
    return x ^ (x >> 31)


def stream_id(seed: int, *tags: int) -> int:
    """Derive a 64-bit stream base from a master seed and integer tags."""
    h = _mix64_int(seed ^ 0x9E3779B97F4A7C15)
    for t in tags:
        h = _mix64_int(h ^ ((t + 0x632BE59BD9B4E019) & _MASK64))
    return h


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift on int64 tensors."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _hash_bits24(base: int, start: int, n: int, device) -> torch.Tensor:
    x = torch.arange(start, start + n, dtype=torch.int64, device=device) + _s64(base)
    x = (x ^ _lsr(x, 30)) * _s64(0xBF58476D1CE4E5B9)
    x = (x ^ _lsr(x, 27)) * _s64(0x94D049BB133111EB)
    x = x ^ _lsr(x, 31)
    return _lsr(x, 40)  # top 24 bits, in [0, 2^24)


def hash_uniform(base: int, n: int, device="cpu", chunk: int = 1 << 26) -> torch.Tensor:
    """n fp32 values uniform on the grid {-1 + k 2^-23 : 0 <= k < 2^24}, element i a pure
    function of (base, i).  Exact in fp32, hence identical on every device."""
    out = torch.empty(n, dtype=torch.float32, device=device)
    for s in range(0, n, chunk):
        m = min(chunk, n - s)
        bits = _hash_bits24(base, s, m, device)
        out[s:s + m] = bits.to(torch.float32) * (2.0 ** -23) - 1.0
    return out


def hash_ints(base: int, n: int, hi: int, device="cpu") -> torch.Tensor:
    """n int32 values uniform-ish on [0, hi) (24 hash bits scaled; hi < 2^24 * 2^7)."""
    bits = _hash_bits24(base, 0, n, device)
    return ((bits * hi) >> 24).to(torch.int32)


@dataclasses.dataclass(frozen=True)
class ModelConfig:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str = "bf16"          # "fp32" | "bf16"  (stored dtype of the matrices)
    rope_theta: float = 10000.0
    rms_eps: float = 1e-6

    @property
    def qkv_out(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16

    def n_params(self) -> int:
        per_layer = (self.qkv_out * self.d_model + self.d_model * self.n_q_heads * self.head_dim
                     + 3 * self.d_ffn * self.d_model)
        return self.n_layers * per_layer + 2 * self.vocab * self.d_model


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    model: Optional[ModelConfig]
    P: int            # prefix length
    K: int            # number of drafts
    T: int            # draft length
    n_cal: int        # calibration-set size
    alphas: tuple     # ascending miscoverage levels
    seed: int
    n_new: int = 0    # scores appended per online step (calibration-only workload)
    n_test: int = 0   # test scores per step           (calibration-only workload)
    n_steps: int = 1


WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", ModelConfig(2, 128, 4, 4, 32, 512, 1024, "fp32"),
                     P=64, K=8, T=32, n_cal=200, alphas=(0.1,), seed=0xA7750001),
    "7b": Workload("7b", ModelConfig(28, 3584, 28, 4, 128, 18944, 152064, "bf16"),
                   P=512, K=16, T=256, n_cal=1000, alphas=(0.1,), seed=0xA7750002),
    "32b": Workload("32b", ModelConfig(64, 5120, 40, 8, 128, 27648, 152064, "bf16"),
                    P=2048, K=64, T=512, n_cal=5000, alphas=(0.05,), seed=0xA7750003),
    "70b": Workload("70b", ModelConfig(80, 8192, 64, 8, 128, 28672, 128256, "bf16"),
                    P=1024, K=32, T=256, n_cal=2000, alphas=(0.1,), seed=0xA7750004),
    "calib": Workload("calib", None, P=0, K=0, T=0, n_cal=1 << 20, alphas=(0.05, 0.2),
                      seed=0xA7750005, n_new=1 << 16, n_test=1 << 16, n_steps=16),
}


# tensor-kind tags for stream_id
_T_EMBED, _T_FNORM, _T_LMHEAD, _T_ANORM, _T_WQKV, _T_WO, _T_MNORM, _T_WGU, _T_WDOWN = range(9)


def _matrix(base: int, rows: int, cols: int, amp: float, dtype, device) -> torch.Tensor:
    u = hash_uniform(base, rows * cols, device)
    u.mul_(float(np.float32(amp)))
    return u.view(rows, cols).to(dtype)


def _gain(base: int, n: int, device) -> torch.Tensor:
    return hash_uniform(base, n, device).mul_(0.1).add_(1.0)


def make_weights(cfg: ModelConfig, seed: int, device="cpu",
                 n_layers: Optional[int] = None) -> Dict[str, object]:
    """Random-init weights in their stored dtype.

    Returns {"tok_embed","final_norm","lm_head": tensor, "attn_norm","wqkv","wo",
    "ffn_norm","w_gate_up","w_down": list of per-layer tensors}.  Matrices are
    [out_features, in_features] row-major.  Norm gains are always fp32.
    ``n_layers`` (default cfg.n_layers) lets a test build the first few layers only; the
    1/sqrt(2L) branch scale always uses cfg.n_layers so a slice matches the full model.
    """
    L = cfg.n_layers if n_layers is None else n_layers
    d, hd, F, V = cfg.d_model, cfg.head_dim, cfg.d_ffn, cfg.vocab
    dt = cfg.torch_dtype
    branch = 1.0 / math.sqrt(2.0 * max(cfg.n_layers, 1))
    w: Dict[str, object] = {
        "tok_embed": _matrix(stream_id(seed, _T_EMBED), V, d, math.sqrt(3.0), dt, device),
        "final_norm": _gain(stream_id(seed, _T_FNORM), d, device),
        "lm_head": _matrix(stream_id(seed, _T_LMHEAD), V, d, math.sqrt(3.0 / d), dt, device),
    }
    names = ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")
    for n in names:
        w[n] = []
    qd = cfg.n_q_heads * hd
    for l in range(L):
        w["attn_norm"].append(_gain(stream_id(seed, _T_ANORM, l), d, device))
        w["wqkv"].append(_matrix(stream_id(seed, _T_WQKV, l), cfg.qkv_out, d,
                                 math.sqrt(3.0 / d), dt, device))
        w["wo"].append(_matrix(stream_id(seed, _T_WO, l), d, qd,
                               math.sqrt(3.0 / qd) * branch, dt, device))
        w["ffn_norm"].append(_gain(stream_id(seed, _T_MNORM, l), d, device))
        w["w_gate_up"].append(_matrix(stream_id(seed, _T_WGU, l), 2 * F, d,
                                      math.sqrt(3.0 / d), dt, device))
        w["w_down"].append(_matrix(stream_id(seed, _T_WDOWN, l), d, F,
                                   math.sqrt(3.0 / F) * branch, dt, device))
    return w


def make_token_ids(vocab: int, P: int, K: int, T: int, seed: int, device="cpu"):
    """(prefix_ids int32 [P], draft_ids int32 [K, T]) uniform over the vocabulary."""
    prefix = hash_ints(stream_id(seed, 100), P, vocab, device)
    drafts = hash_ints(stream_id(seed, 101), K * T, vocab, device).view(K, T)
    return prefix, drafts


def lognormal_scores(n: int, seed: int, mu: float = 0.0, sigma: float = 1.0) -> np.ndarray:
    """n fp32 scores ~ lognormal(mu, sigma): exp of an fp64 normal draw, rounded once."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return np.exp(mu + sigma * rng.standard_normal(n)).astype(np.float32)
