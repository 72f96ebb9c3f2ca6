"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds no arithmetic of the three kernels (no factorisation, no
3mm): it only synthesises matrices.  The paper takes its inputs from the
benchmark suite's own array initialisers, which are not reproduced here; these
generators stand in for them with the paper's shapes (Section "Linear Algebra
Benchmarks": N = 2000 / 4000 for LU and Cholesky, five free dimensions for 3mm).

Random entries come from a counter-based generator, so element (i, j) of
matrix ``tag`` under ``seed`` is a pure function of (seed, tag, i*cols + j) and
does not depend on generation order: the splitmix64 output function applied to
the counter, top 53 bits scaled to [0, 1), mapped to [-1, 1).
"""
from __future__ import annotations

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on an array of uint64 counters (wrap-around arithmetic)."""
    with np.errstate(over="ignore"):
        z = (z + _GOLDEN).astype(np.uint64)
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def _stream_base(seed: int, tag: int) -> np.uint64:
    s = _mix64(np.array([np.uint64(seed & 0xFFFFFFFFFFFFFFFF)], dtype=np.uint64))
    with np.errstate(over="ignore"):
        t = _mix64(s ^ (np.uint64(tag & 0xFFFFFFFFFFFFFFFF) * _GOLDEN))
    return t[0]


def random_bits(seed: int, tag: int, count: int) -> np.ndarray:
    """count uint64 words, word c = mix(base(seed, tag) + c * golden)."""
    base = _stream_base(seed, tag)
    idx = np.arange(count, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix64(base + idx * _GOLDEN)


def uniform_matrix(seed: int, tag: int, rows: int, cols: int) -> np.ndarray:
    """rows x cols fp64 matrix with entries uniform in [-1, 1), row-major."""
    bits = random_bits(seed, tag, rows * cols)
    u = (bits >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
    return (2.0 * u - 1.0).reshape(rows, cols)


def integer_matrix(seed: int, tag: int, rows: int, cols: int, lo: int = -3, hi: int = 3) -> np.ndarray:
    """rows x cols fp64 matrix with integer entries uniform in {lo..hi} (exactly representable)."""
    bits = random_bits(seed, tag, rows * cols)
    span = np.uint64(hi - lo + 1)
    return ((bits >> np.uint64(33)) % span).astype(np.float64).reshape(rows, cols) + float(lo)


def _gram(M: np.ndarray) -> np.ndarray:
    """M*M^T/N, exactly symmetric (input synthesis only; any trusted matmul will do)."""
    n = M.shape[0]
    S = (M @ M.T) / float(n)
    return np.tril(S) + np.tril(S, -1).T


def spd_matrix(n: int, seed: int) -> np.ndarray:
    """Symmetric positive-definite A = M*M^T/N + I, M uniform in [-1, 1) (Cholesky input)."""
    A = _gram(uniform_matrix(seed, 0, n, n))
    A[np.diag_indices(n)] += 1.0
    return A


def diag_dominant_matrix(n: int, seed: int) -> np.ndarray:
    """A = M*M^T/N + N*I: diagonally dominant, so LU without pivoting is stable (LU input)."""
    A = _gram(uniform_matrix(seed, 0, n, n))
    A[np.diag_indices(n)] += float(n)
    return A


def general_dominant_matrix(n: int, seed: int) -> np.ndarray:
    """Non-symmetric A = M + N*I with M uniform in [-1, 1): strictly row-diagonally dominant."""
    A = uniform_matrix(seed, 1, n, n)
    A[np.diag_indices(n)] += float(n)
    return A


def mm3_operands(seed: int, ni: int, nk: int, nj: int, nm: int, nl: int):
    """A (ni x nk), B (nk x nj), C (nj x nm), D (nm x nl), uniform in [-1, 1)."""
    return (uniform_matrix(seed, 10, ni, nk), uniform_matrix(seed, 11, nk, nj),
            uniform_matrix(seed, 12, nj, nm), uniform_matrix(seed, 13, nm, nl))


def mm3_integer_operands(seed: int, ni: int, nk: int, nj: int, nm: int, nl: int):
    """Same shapes with integer entries in {-3..3}: every partial sum of 3mm is then exact."""
    return (integer_matrix(seed, 10, ni, nk), integer_matrix(seed, 11, nk, nj),
            integer_matrix(seed, 12, nj, nm), integer_matrix(seed, 13, nm, nl))


def min_index_matrix(n: int) -> np.ndarray:
    """A[i][j] = min(i, j) + 1 (0-based): SPD with all-ones triangular factors, exact in fp64/fp32."""
    i = np.arange(n, dtype=np.float64)
    return np.minimum.outer(i, i) + 1.0


# The workload shapes named by the benchmark configuration.
MM3_SMALL = dict(ni=128, nk=128, nj=128, nm=128, nl=128)
MM3_EXTRALARGE = dict(ni=1600, nk=2000, nj=1800, nm=2400, nl=2200)
MM3_EXTRALARGE_PAPER_ORDER = dict(ni=1600, nk=1800, nj=2000, nm=2200, nl=2400)
MM3_LARGE_PAPER_ORDER = dict(ni=800, nk=900, nj=1000, nm=1100, nl=1200)
