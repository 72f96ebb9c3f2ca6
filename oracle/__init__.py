"""CPU oracle (test infrastructure only) for 3mm, LU without pivoting, Cholesky, and solves with the factors.

The arithmetic lives in ``dla_oracle.c`` (plain fp64 loop nests that follow the
problem statements in the paper's Section "Linear Algebra Benchmarks").  This
module only compiles that file with gcc, loads it with ctypes and marshals
numpy arrays.  It imports nothing from the HIP package and must never be used
by the product path: only ``tests/``, the smoke check and the benchmark's
``cpu_baseline`` leg may call it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "dla_oracle.c"
_LIB = _HERE / "libdla_oracle.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (-O3, AVX2, OpenMP; strict fp: no fast-math, no fma contraction)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".so.tmp{os.getpid()}")
        cmd = ["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", str(tmp), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(str(_LIB))
    dp = ctypes.POINTER(ctypes.c_double)
    i64 = ctypes.c_int64
    lib.oracle_num_threads.restype = ctypes.c_int
    lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
    lib.oracle_mm3.argtypes = [dp] * 7 + [i64] * 5
    lib.oracle_mm3.restype = None
    lib.oracle_lu.argtypes = [dp, i64, i64]
    lib.oracle_lu.restype = i64
    lib.oracle_cholesky.argtypes = [dp, i64, i64]
    lib.oracle_cholesky.restype = i64
    lib.oracle_lu_residual.argtypes = [dp, i64, dp, i64, i64]
    lib.oracle_lu_residual.restype = ctypes.c_double
    lib.oracle_cholesky_residual.argtypes = [dp, i64, dp, i64, i64]
    lib.oracle_cholesky_residual.restype = ctypes.c_double
    lib.oracle_lu_apply.argtypes = [dp, i64, i64, dp, dp, dp]
    lib.oracle_cholesky_apply.argtypes = [dp, i64, i64, dp, dp, dp]
    lib.oracle_matvec.argtypes = [dp, i64, i64, i64, dp, dp]
    lib.oracle_symv_lower.argtypes = [dp, i64, i64, dp, dp]
    lib.oracle_lu_solve.argtypes = [dp, i64, i64, dp, i64, i64]
    lib.oracle_lu_solve.restype = None
    lib.oracle_cholesky_solve.argtypes = [dp, i64, i64, dp, i64, i64]
    lib.oracle_cholesky_solve.restype = None
    _lib = lib
    return lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _dense(a, name: str) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float64)
    if a.ndim != 2:
        raise ValueError(f"{name} must be a matrix")
    return a


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(t: int) -> None:
    _load().oracle_set_num_threads(int(t))


def mm3(A, B, C, D, return_intermediates: bool = False):
    """G = (A*B)*(C*D) by three plain products; optionally also E = A*B and F = C*D."""
    A, B, C, D = (_dense(x, n) for x, n in ((A, "A"), (B, "B"), (C, "C"), (D, "D")))
    ni, nk = A.shape
    nk2, nj = B.shape
    nj2, nm = C.shape
    nm2, nl = D.shape
    if nk != nk2 or nj != nj2 or nm != nm2:
        raise ValueError("3mm inner dimensions do not match")
    E = np.empty((ni, nj))
    F = np.empty((nj, nl))
    G = np.empty((ni, nl))
    _load().oracle_mm3(_p(A), _p(B), _p(C), _p(D), _p(E), _p(F), _p(G), ni, nk, nj, nm, nl)
    return (G, E, F) if return_intermediates else G


def lu(A):
    """In-place-style LU without pivoting of a copy of A: returns (LU, info).

    LU holds unit-lower L below the diagonal and U on and above it; info is 0
    or the 1-based index of the first zero pivot.
    """
    a = np.array(A, dtype=np.float64, order="C", copy=True)
    if a.ndim != 2 or a.shape[0] != a.shape[1]:
        raise ValueError("A must be square")
    info = _load().oracle_lu(_p(a), a.shape[0], a.shape[1])
    return a, int(info)


def cholesky(A):
    """Cholesky factor of the symmetric matrix given by A's lower triangle: returns (L, info)."""
    a = np.array(A, dtype=np.float64, order="C", copy=True)
    if a.ndim != 2 or a.shape[0] != a.shape[1]:
        raise ValueError("A must be square")
    info = _load().oracle_cholesky(_p(a), a.shape[0], a.shape[1])
    return a, int(info)


def lu_residual(A0, LU) -> float:
    A0 = _dense(A0, "A0")
    LU = _dense(LU, "LU")
    n = A0.shape[0]
    return float(_load().oracle_lu_residual(_p(A0), A0.shape[1], _p(LU), LU.shape[1], n))


def cholesky_residual(A0, L) -> float:
    A0 = _dense(A0, "A0")
    L = _dense(L, "L")
    n = A0.shape[0]
    return float(_load().oracle_cholesky_residual(_p(A0), A0.shape[1], _p(L), L.shape[1], n))


def lu_apply(LU, x):
    """y = L*(U*x) from an in-place LU result."""
    LU = _dense(LU, "LU")
    n = LU.shape[0]
    x = np.ascontiguousarray(x, dtype=np.float64)
    tmp = np.empty(n)
    y = np.empty(n)
    _load().oracle_lu_apply(_p(LU), LU.shape[1], n, _p(x), _p(tmp), _p(y))
    return y


def cholesky_apply(L, x):
    """y = L*(L^T*x) from the lower triangle of L."""
    L = _dense(L, "L")
    n = L.shape[0]
    x = np.ascontiguousarray(x, dtype=np.float64)
    tmp = np.empty(n)
    y = np.empty(n)
    _load().oracle_cholesky_apply(_p(L), L.shape[1], n, _p(x), _p(tmp), _p(y))
    return y


def matvec(A, x):
    A = _dense(A, "A")
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.empty(A.shape[0])
    _load().oracle_matvec(_p(A), A.shape[1], A.shape[0], A.shape[1], _p(x), _p(y))
    return y


def symv_lower(A, x):
    """y = S*x with S the symmetric matrix whose lower triangle is A's."""
    A = _dense(A, "A")
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.empty(A.shape[0])
    _load().oracle_symv_lower(_p(A), A.shape[1], A.shape[0], _p(x), _p(y))
    return y


def _rhs(B, n: int):
    b = np.array(B, dtype=np.float64, order="C", copy=True)
    vec = b.ndim == 1
    if vec:
        b = b.reshape(n, 1)
    if b.ndim != 2 or b.shape[0] != n:
        raise ValueError("B must have as many rows as the factor")
    return b, vec


def lu_solve(LU, B):
    """X with (L*U)*X = B, from an in-place LU result: forward substitution with unit-lower L, backward with U."""
    LU = _dense(LU, "LU")
    n = LU.shape[0]
    b, vec = _rhs(B, n)
    _load().oracle_lu_solve(_p(LU), n, LU.shape[1], _p(b), b.shape[1], b.shape[1])
    return b[:, 0] if vec else b


def cholesky_solve(L, B):
    """X with (L*L^T)*X = B, from the lower triangle of L: forward with L, backward with L^T."""
    L = _dense(L, "L")
    n = L.shape[0]
    b, vec = _rhs(B, n)
    _load().oracle_cholesky_solve(_p(L), n, L.shape[1], _p(b), b.shape[1], b.shape[1])
    return b[:, 0] if vec else b
