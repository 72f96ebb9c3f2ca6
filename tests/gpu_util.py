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


def oracle_product(oracle, X, Y) -> np.ndarray:
    """X * Y by the oracle's plain triple loop: the E of a 3mm whose second product is empty-sized."""
    X, Y = np.ascontiguousarray(X), np.ascontiguousarray(Y)
    return oracle.mm3(X, Y, np.zeros((Y.shape[1], 1)), np.zeros((1, 1)), return_intermediates=True)[1]
