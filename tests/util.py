"""Helpers shared by the GPU parity tests (no method arithmetic here)."""
import numpy as np
import torch


def weights_to_numpy(w):
    """Stored weight values as fp32 numpy arrays (bf16 -> fp32 is exact); the oracle widens to fp64."""
    conv = lambda t: t.detach().float().cpu().numpy()
    return {k: ([conv(t) for t in v] if isinstance(v, list) else conv(v)) for k, v in w.items()}


def dev(x, dtype=None):
    t = torch.as_tensor(x)
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda().contiguous()


def ws(nbytes):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")


def announce(*what):
    """Name the case before the GPU step runs, flushed, so a lost box still tells which case it was."""
    print("[case]", *what, flush=True)
