"""Comparison metrics used by the parity tests (plain numpy, no kernel arithmetic).

max_rel_err: the gating elementwise error.  A literal elementwise relative
error is unbounded for entries that happen to be near zero (3mm outputs are
random-sign sums), so the denominator is floored at the RMS of the expected
entries:  max_ij |x - y| / max(|y|, rms(y)).
"""
import numpy as np

EPS64 = 2.0 ** -52
EPS32 = 2.0 ** -23


def max_rel_err(got, want, mask=None) -> float:
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if mask is not None:
        got = got[mask]
        want = want[mask]
    if want.size == 0:
        return 0.0
    floor = float(np.sqrt(np.mean(want * want)))
    if floor == 0.0:
        floor = 1.0
    return float(np.max(np.abs(got - want) / np.maximum(np.abs(want), floor)))


def fro_rel_err(got, want) -> float:
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    den = float(np.linalg.norm(want))
    num = float(np.linalg.norm(got - want))
    return num / den if den > 0 else num


def lower_mask(n: int, strict: bool = False):
    return np.tril(np.ones((n, n), dtype=bool), -1 if strict else 0)
