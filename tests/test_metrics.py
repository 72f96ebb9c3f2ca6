"""The parity gates themselves, checked on the CPU with mistakes planted in the oracle's own factors.

The gate for an in-place LU result compares L, the strict upper part of U and the diagonal each against
its own floor.  On the benchmark's diagonally dominant inputs one floor over the whole array (the RMS is
set by the N-sized diagonal) would let a factor with a whole block update missing pass by a small margin;
these tests pin that the per-part gate rejects such a factor by at least two orders of magnitude.
"""
import numpy as np
import pytest

from paper_2309_07235_amd import inputs
from tests.metrics import cholesky_rel_err, lu_rel_err, lu_rel_err_parts, max_rel_err

TOL64 = 1e-9
NB = 128


def _lu_with_one_block_update_missing(lu, bi, bj, bk):
    """The factor a blocked right-looking LU would store if block (bi, bj) of the trailing matrix had missed
    step bk's rank-128 update  A[bi][bj] -= L[bi][bk] * U[bk][bj]  (bk < min(bi, bj)) and nothing after it
    had been recomputed: the block keeps the product it should have lost, carried through the solve that
    finishes it (U[bj][bj]^-1 from the right for a block of L, L[bi][bi]^-1 from the left for a block of U)."""
    out = lu.copy()
    r = slice(bi * NB, (bi + 1) * NB)
    c = slice(bj * NB, (bj + 1) * NB)
    k = slice(bk * NB, (bk + 1) * NB)
    extra = lu[r, k] @ lu[k, c]
    if bi > bj:    # a block of L
        ujj = np.triu(lu[c, c])
        out[r, c] += np.linalg.solve(ujj.T, extra.T).T
    elif bi < bj:  # a block of U
        lii = np.tril(lu[r, r], -1) + np.eye(NB)
        out[r, c] += np.linalg.solve(lii, extra)
    else:          # a diagonal block: to first order the upper part moves by L^-1 * extra, the lower by extra * U^-1
        lii = np.tril(lu[r, r], -1) + np.eye(NB)
        uii = np.triu(lu[r, r])
        d = np.linalg.solve(lii, extra)
        out[r, c] += np.triu(d) + np.tril(np.linalg.solve(uii.T, d.T).T, -1)
    return out


@pytest.mark.parametrize("n", [2000, 4000])
def test_lu_gate_rejects_a_missing_block_update(oracle, n):
    A = inputs.diag_dominant_matrix(n, 5)
    want, info = oracle.lu(A)
    assert info == 0
    assert lu_rel_err(want, want) == 0.0
    nblk = n // NB
    for bi, bj, bk in ((nblk - 1, 3, 1), (3, nblk - 1, 1), (nblk - 2, nblk - 2, 0), (nblk // 2, nblk // 2 - 1, 2)):
        bad = _lu_with_one_block_update_missing(want, bi, bj, bk)
        parts = lu_rel_err_parts(bad, want)
        assert max(parts.values()) >= 100 * TOL64, (n, bi, bj, bk, parts)
        hit = "L" if bi > bj else "U"
        if bi != bj:
            assert parts[hit] >= 100 * TOL64, (n, bi, bj, bk, parts)
    # what one floor over the whole array makes of the same mistake: within an order of the bar at N = 4000
    bad = _lu_with_one_block_update_missing(want, nblk - 1, 3, 1)
    assert max_rel_err(bad, want) < lu_rel_err(bad, want) / 1e3


def test_lu_gate_is_relative_within_each_part(oracle):
    n = 600
    A = inputs.diag_dominant_matrix(n, 7)
    want, _ = oracle.lu(A)
    low = np.tril(np.ones((n, n), dtype=bool), -1)
    rms_l = np.sqrt(np.mean(want[low] ** 2))
    # a relative perturbation of one typical L entry shows at its own size ...
    i, j = np.argwhere(low & (np.abs(want) > rms_l))[0]
    bad = want.copy()
    bad[i, j] *= 1.0 + 1e-6
    assert 0.9e-6 <= lu_rel_err_parts(bad, want)["L"] <= 1.1e-6
    assert lu_rel_err_parts(bad, want)["U"] == 0.0 and lu_rel_err_parts(bad, want)["diag"] == 0.0
    # ... and an absolute one far below the diagonal's size still fails the L part
    bad = want.copy()
    bad[i, j] += 1e-11
    assert lu_rel_err(bad, want) > 1e-7 and max_rel_err(bad, want) < 1e-11
    # rounding-sized differences pass
    bad = want * (1.0 + 4 * np.finfo(np.float64).eps)
    assert lu_rel_err(bad, want) <= 1e-14


def test_cholesky_gate_rejects_a_missing_block_update(oracle):
    n = 2000
    A = inputs.spd_matrix(n, 5)
    want, info = oracle.cholesky(A)
    assert info == 0 and cholesky_rel_err(want, want) == 0.0
    nblk = n // NB
    bi, bj, bk = nblk - 1, 4, 2
    r, c, k = (slice(b * NB, (b + 1) * NB) for b in (bi, bj, bk))
    bad = want.copy()
    # block (bi, bj) missed  A[bi][bj] -= L[bi][bk] * L[bj][bk]^T ; the panel solve then divides by L[bj][bj]^T
    extra = want[r, k] @ want[c, k].T
    bad[r, c] += np.linalg.solve(np.tril(want[c, c]), extra.T).T
    assert cholesky_rel_err(bad, want) >= 100 * TOL64
    # a wrong diagonal entry is gated against the diagonal's floor
    bad = want.copy()
    bad[17, 17] *= 1.0 + 1e-7
    assert 0.9e-7 <= cholesky_rel_err(bad, want) <= 1.1e-7
