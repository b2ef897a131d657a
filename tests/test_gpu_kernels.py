"""Stage-level parity: the MFMA GEMM, the fused LM-head log-softmax-gather and the shared-prefix
attention, each against a plain float64 statement of the same operation."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import atts_oracle as O
from synth import hash_uniform, stream_id
from util import announce, dev, ws

pytestmark = pytest.mark.gpu


def _rand(shape, seed, dtype, scale=1.0):
    n = int(np.prod(shape))
    return (hash_uniform(stream_id(seed, 1), n) * scale).view(*shape).to(dtype)


# ------------------------------------------------------------------------------------ GEMM
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape", [(1, 1, 8), (33, 70, 72), (300, 200, 136), (257, 513, 1000), (128, 128, 64),
                                   (3584, 3600, 264),
                                   # aligned bf16 shapes with more 384-row tiles than compute units: workgroups walk two or
                                   # three tiles each, some one fewer than others (510 and 700 tiles)
                                   (1152, 43520, 768), (768, 89600, 832),
                                   # at most 16 rows: the weight-streaming kernel (bf16), ragged columns and k-step counts
                                   (1, 1, 32), (4, 100, 96), (7, 4608, 256), (16, 33, 2080), (16, 530, 3584), (3, 48, 18944)])
def test_gemm_nt_matches_float64_matmul(dtype, shape):
    import paper_2509_15148_amd as A
    M, N, Kd = shape
    announce("gemm", dtype, shape)
    a, w = _rand((M, Kd), 11, dtype), _rand((N, Kd), 12, dtype)
    c = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    A.atts_gemm_nt(a.cuda(), w.cuda(), c)
    torch.cuda.synchronize()
    ref = a.double().numpy() @ w.double().numpy().T
    assert np.allclose(c.cpu().numpy(), ref, rtol=1e-5, atol=2e-5 * math.sqrt(Kd))


def test_gemm_aligned_last_tile_rows_in_a_second_launch():
    """27 x 38 tiles of 384 x 256 = 1026 = four rounds of 256 and two tiles over: the aligned bf16 path gives the last
    tile row to a launch of its own with 128-row tiles (26 x 38 = 988 tiles in four rounds, then 384 rows as 114 small
    tiles).  Every element against the float64 product."""
    import paper_2509_15148_amd as A
    M, N, Kd = 10368, 9728, 768
    announce("gemm tail launch", (M, N, Kd))
    a, w = _rand((M, Kd), 21, torch.bfloat16), _rand((N, Kd), 22, torch.bfloat16)
    c = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    A.atts_gemm_nt(a.cuda(), w.cuda(), c)
    torch.cuda.synchronize()
    ref = a.double().numpy() @ w.double().numpy().T
    assert np.allclose(c.cpu().numpy(), ref, rtol=1e-5, atol=2e-5 * math.sqrt(Kd))


def test_gemm_aligned_shapes_sweep():
    """Seeded sweep over shapes the aligned bf16 kernel takes (rows a multiple of 256 or 384, columns of 256, inner
    dimension of 64 from 768 up): tile counts below and above the number of compute units, partly filled last rounds of
    the tile walk, both tile heights.  Every element against the float64 product."""
    import paper_2509_15148_amd as A
    rng = np.random.default_rng(15148)
    for case in range(12):
        M = int(rng.choice([256, 384, 768, 1152, 1280, 1536, 2304, 3072, 4224]))
        N = 256 * int(rng.integers(1, 90))
        Kd = 64 * int(rng.choice([12, 13, 16, 24, 31]))
        announce("gemm aligned", case, (M, N, Kd))
        a, w = _rand((M, Kd), 300 + case, torch.bfloat16), _rand((N, Kd), 400 + case, torch.bfloat16)
        c = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        A.atts_gemm_nt(a.cuda(), w.cuda(), c)
        torch.cuda.synchronize()
        ref = a.double().numpy() @ w.double().numpy().T
        assert np.allclose(c.cpu().numpy(), ref, rtol=1e-5, atol=2e-5 * math.sqrt(Kd)), (M, N, Kd)


def test_gemm_few_rows_random_shapes():
    """Seeded sweep over the shapes the weight-streaming kernel serves (1..16 rows, any column count, inner
    dimension a multiple of 32 up to several K slices), against the float64 product."""
    import paper_2509_15148_amd as A
    rng = np.random.default_rng(2509)
    for case in range(24):
        M = int(rng.integers(1, 17))
        N = int(rng.choice([1, 15, 16, 17, 31, 32, 33, 100, 255, 256, 1000, 3584, 4608]))
        Kd = 32 * int(rng.choice([1, 2, 3, 7, 8, 9, 16, 17, 63, 112, 129]))
        announce("gemm few rows", case, (M, N, Kd))
        a, w = _rand((M, Kd), 100 + case, torch.bfloat16), _rand((N, Kd), 200 + case, torch.bfloat16)
        c = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        A.atts_gemm_nt(a.cuda(), w.cuda(), c)
        torch.cuda.synchronize()
        ref = a.double().numpy() @ w.double().numpy().T
        assert np.allclose(c.cpu().numpy(), ref, rtol=1e-5, atol=2e-5 * math.sqrt(Kd)), (M, N, Kd)


def test_gemm_rejects_unaligned_k():
    import paper_2509_15148_amd as A
    a = torch.zeros(4, 12, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(A.AttsError) as e:
        A.atts_gemm_nt(a, a, torch.zeros(4, 4, device="cuda"))
    assert e.value.code == A.ERR_SHAPE


# ------------------------------------------------------------------------------------ LM head
@pytest.mark.parametrize("dtype,tol", [(torch.float32, 1e-4), (torch.bfloat16, 1e-3)])
@pytest.mark.parametrize("shape", [(1, 16, 7), (37, 128, 1000), (256, 128, 1024), (130, 264, 5003), (4096, 256, 19008),
                                   # scoring rows a multiple of 256, vocabulary of 384, inner dimension of 64 from 768 up: the
                                   # bf16 product is taken with the operands exchanged (vocabulary entries as rows); 300 and 30
                                   # tiles, the second with a single column of tiles
                                   (1280, 768, 23040), (256, 1344, 11520)])
def test_lmhead_logprobs_matches_log_softmax_gather(dtype, tol, shape):
    """lp = z[target] - logsumexp(z) without materialising z; logits scaled to a spread of several
    units so that the running-max logic matters."""
    import paper_2509_15148_amd as A
    B, d, V = shape
    announce("lmhead", dtype, shape)
    x = _rand((B, d), 21, dtype, scale=2.0)
    w = _rand((V, d), 22, dtype, scale=4.0 / math.sqrt(d))
    tgt = torch.from_numpy(np.random.default_rng(3).integers(0, V, B).astype(np.int32))
    tgt[0], tgt[-1] = V - 1, 0
    lp = torch.full((B,), float("nan"), dtype=torch.float32, device="cuda")
    A.atts_lmhead_logprobs(x.cuda(), w.cuda(), tgt.cuda(), lp, ws(A.atts_lmhead_workspace_bytes(B, V)))
    torch.cuda.synchronize()
    z = x.double().numpy() @ w.double().numpy().T
    ref = O.log_softmax(z)[np.arange(B), tgt.numpy()]
    got = lp.cpu().numpy()
    assert np.abs(got - ref).max() <= tol, np.abs(got - ref).max()
    assert np.all(got <= 1e-6)


# ------------------------------------------------------------------------------------ attention
def _tree_attention_reference(qkv, P, K, T, nq, nkv, hd):
    """K independent causal sequences [prefix ; draft k] through torch's float64 SDPA."""
    R = P + K * T
    q, k, v = qkv.double().split([nq * hd, nkv * hd, nkv * hd], -1)
    out = torch.zeros(R, nq * hd, dtype=torch.float64)

    def run(rows):
        n = len(rows)
        o = F.scaled_dot_product_attention(q[rows].view(n, nq, hd).transpose(0, 1)[None],
                                           k[rows].view(n, nkv, hd).transpose(0, 1)[None],
                                           v[rows].view(n, nkv, hd).transpose(0, 1)[None],
                                           is_causal=True, enable_gqa=True)
        return o[0].transpose(0, 1).reshape(n, nq * hd)

    pre = torch.arange(P)
    out[:P] = run(pre)
    for kk in range(K):
        rows = torch.cat([pre, P + kk * T + torch.arange(T)])
        out[P + kk * T: P + (kk + 1) * T] = run(rows)[P:]
    return out.numpy()


@pytest.mark.parametrize("dtype,shape,tol", [
    (torch.float32, (64, 8, 32, 4, 4, 32), 2e-5),          # the tiny workload's shape
    (torch.float32, (5, 3, 7, 6, 2, 16), 2e-5),
    (torch.bfloat16, (9, 2, 5, 4, 2, 64), 1.5e-2),         # simple kernel in bf16
    (torch.bfloat16, (70, 3, 45, 4, 2, 128), 1.5e-2),      # MFMA kernel, nothing aligned
    (torch.bfloat16, (1, 4, 1, 2, 1, 128), 1.5e-2),
    (torch.bfloat16, (130, 5, 17, 8, 8, 128), 1.5e-2),     # several drafts inside one query tile
    (torch.bfloat16, (512, 4, 256, 7, 1, 128), 1.5e-2),    # aligned, GQA group 7
    (torch.bfloat16, (200, 0, 1, 2, 2, 128), 1.5e-2),      # prefix only
    (torch.bfloat16, (512, 16, 256, 28, 4, 128), 1.5e-2),  # the 7B step's launch: 256-row query tiles, 504 workgroups
    (torch.bfloat16, (200, 21, 200, 16, 2, 128), 1.5e-2),  # the same kernel (288 workgroups), drafts and prefix not aligned to its tiles
])
def test_shared_prefix_attention(dtype, shape, tol):
    import paper_2509_15148_amd as A
    P, K, T, nq, nkv, hd = shape
    announce("attention", dtype, shape)
    R = P + K * T
    qkv = _rand((R, (nq + 2 * nkv) * hd), 31, dtype, scale=1.5)
    out = torch.full((R, nq * hd), float("nan"), dtype=dtype, device="cuda")
    wsb = A.atts_attention_workspace_bytes(dtype, R, nkv, hd)
    A.atts_attention_shared_prefix(qkv.cuda(), out, P, K, T, nq, nkv, hd, ws(wsb) if wsb else None)
    torch.cuda.synchronize()
    ref = _tree_attention_reference(qkv, P, K, T, nq, nkv, hd)
    err = np.abs(out.float().cpu().numpy() - ref).max()
    assert err <= tol, err
