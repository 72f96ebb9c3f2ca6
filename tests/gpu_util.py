"""Helpers for the GPU parity tests: device transfer and named progress lines."""
import sys

import numpy as np


def announce(msg: str) -> None:
    """Print (and flush) what is about to run so a fault can be traced to its case."""
    print(f"[case] {msg}", file=sys.stderr, flush=True)


def to_device(a: np.ndarray, dtype=None):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def to_host(t) -> np.ndarray:
    import torch
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()
