"""The LM-head entry point that allocates nothing (its scratch is a device array inside the library) against the
workspace form of the same stage: same kernels, so the log-probs must be equal bit for bit, and to the oracle's
log-softmax-gather within the stage tolerance.  Two calls in a row on the one shared array, the second smaller."""
import math

import numpy as np
import pytest
import torch

from oracle import atts_oracle as O
from util import announce, ws

pytestmark = pytest.mark.gpu


def _inputs(B, d, V, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    x = (torch.randn(B, d, generator=g) * 2.0).to(dtype)
    w = (torch.randn(V, d, generator=g) * (4.0 / math.sqrt(d))).to(dtype)
    tgt = torch.randint(0, V, (B,), generator=g, dtype=torch.int32)
    tgt[0], tgt[-1] = V - 1, 0
    return x, w, tgt


@pytest.mark.parametrize("dtype,tol", [(torch.bfloat16, 1e-3), (torch.float32, 1e-4)])
def test_static_scratch_lmhead_equals_the_workspace_form(dtype, tol):
    import paper_2509_15148_amd as A
    for B, d, V in ((700, 256, 19008), (130, 264, 5003)):          # the second call is smaller: stale partials of the first
        announce("lmhead static scratch", dtype, (B, d, V))       # stay in the array and must not be read
        x, w, tgt = _inputs(B, d, V, dtype, seed=B)
        xd, wd, td = x.cuda(), w.cuda(), tgt.cuda()
        ref = torch.full((B,), float("nan"), dtype=torch.float32, device="cuda")
        A.atts_lmhead_logprobs(xd, wd, td, ref, ws(A.atts_lmhead_workspace_bytes(B, V)))
        got = torch.full((B,), float("nan"), dtype=torch.float32, device="cuda")
        A.atts_lmhead_logprobs_static(xd, wd, td, got)
        torch.cuda.synchronize()
        assert torch.equal(got, ref)
        z = x.double().numpy() @ w.double().numpy().T
        want = O.log_softmax(z)[np.arange(B), tgt.numpy()]
        assert np.abs(got.cpu().numpy() - want).max() <= tol


def test_static_scratch_limit_is_an_error_before_any_launch():
    import paper_2509_15148_amd as A
    B, d, V = 4096, 128, 152064                                     # 4096 rows x 2376 partials x 8 B > 16 MiB
    assert A.atts_lmhead_workspace_bytes(B, V) > 16 << 20
    x = torch.zeros(B, d, dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(V, d, dtype=torch.bfloat16, device="cuda")
    tgt = torch.zeros(B, dtype=torch.int32, device="cuda")
    lp = torch.full((B,), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(A.AttsError) as e:
        A.atts_lmhead_logprobs_static(x, w, tgt, lp)
    assert e.value.code == A.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((lp == 7.0).all())                                  # nothing ran
