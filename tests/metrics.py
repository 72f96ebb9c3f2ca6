"""Comparison metrics used by the parity tests (plain numpy, no kernel arithmetic).

max_rel_err: the gating elementwise error.  A literal elementwise relative
error is unbounded for entries that happen to be near zero (3mm outputs are
random-sign sums), so the denominator is floored at the RMS of the expected
entries:  max_ij |x - y| / max(|y|, rms(y)).

A factor stored in place holds parts of very different magnitude: for the
diagonally dominant LU inputs the diagonal of U is about N, the strict upper
part of U about 1e-2 and L about 1e-6.  One floor over the whole array would
be set by the diagonal alone and leave L checked to percents only, so the
factor metrics below gate every part against its own floor.
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


def _parts(n: int):
    low = np.tril(np.ones((n, n), dtype=bool), -1)
    return low, low.T, np.eye(n, dtype=bool)


def lu_rel_err_parts(got, want) -> dict:
    """In-place LU result against the expected one: max_rel_err of the strict lower part (L), the strict
    upper part (U without its diagonal) and the diagonal (the pivots), each with its own floor."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    low, up, dia = _parts(want.shape[0])
    return {"L": max_rel_err(got, want, low), "U": max_rel_err(got, want, up), "diag": max_rel_err(got, want, dia)}


def lu_rel_err(got, want) -> float:
    """The gating figure for an in-place LU result: the worst of its three parts."""
    return max(lu_rel_err_parts(got, want).values())


def cholesky_rel_err(got, want) -> float:
    """Lower-triangular factor against the expected one: the worse of the strict lower part and the
    diagonal, each with its own floor (the upper triangle is checked for exact zeros elsewhere)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    low, _, dia = _parts(want.shape[0])
    return max(max_rel_err(got, want, low), max_rel_err(got, want, dia))


def fro_rel_err(got, want) -> float:
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    den = float(np.linalg.norm(want))
    num = float(np.linalg.norm(got - want))
    return num / den if den > 0 else num


def lower_mask(n: int, strict: bool = False):
    return np.tril(np.ones((n, n), dtype=bool), -1 if strict else 0)
