"""GPU parity of lu_solve / cholesky_solve (and the A^T*B product they use) against the CPU oracle."""
import json
import os

import numpy as np
import pytest

from paper_2309_07235_amd import inputs
from tests.gpu_util import announce, oracle_product, to_device, to_host
from tests.metrics import EPS64, max_rel_err

pytestmark = pytest.mark.gpu

TOL64 = 1e-9   # max relative error, denominator floored at the RMS of the expected solution entries
TOL32 = 1e-4
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_worked.json")


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2309_07235_amd import binding
    return binding


def _factor(oracle, kind, n, seed):
    """Matrix and its oracle factor: the solve is then compared on the same factor on both sides."""
    A = inputs.general_dominant_matrix(n, seed) if kind == "lu" else inputs.spd_matrix(n, seed)
    F, info = (oracle.lu if kind == "lu" else oracle.cholesky)(A)
    assert info == 0
    return A, F


def _gpu_solve(B, kind, F, rhs, dtype=None):
    f, b = to_device(F, dtype), to_device(rhs, dtype)
    (B.lu_solve if kind == "lu" else B.cholesky_solve)(f, b)
    return to_host(b)


# sizes span one sub-block, one block, the first ragged block, several blocks with a ragged tail, a last block of
# one row behind four whole ones (odd leading dimension); right-hand sides span one, a ragged slice of 16, one and
# two column blocks per workgroup of the chain's kernel up to its limit (128), and the tiled GEMM's ranges above
@pytest.mark.parametrize("kind", ["lu", "chol"])
@pytest.mark.parametrize("n,nrhs", [(1, 1), (7, 3), (16, 1), (100, 5), (128, 64), (129, 1), (300, 17), (1000, 130),
                                    (517, 260), (1025, 33), (900, 128), (770, 50), (1300, 16)])
def test_solve_matches_oracle(B, oracle, kind, n, nrhs):
    announce(f"solve {kind} n={n} nrhs={nrhs} f64")
    A, F = _factor(oracle, kind, n, 21)
    rhs = inputs.uniform_matrix(22, 3, n, nrhs)
    want = (oracle.lu_solve if kind == "lu" else oracle.cholesky_solve)(F, rhs)
    got = _gpu_solve(B, kind, F, rhs)
    assert max_rel_err(got, want) <= TOL64
    assert np.abs(A @ got - rhs).max() <= 64 * n * EPS64 * np.abs(A).max() * max(np.abs(got).max(), 1e-300)


@pytest.mark.parametrize("kind", ["lu", "chol"])
@pytest.mark.parametrize("n,dtype_name", [(700, "float64"), (129, "float64"), (1025, "float32")])
def test_prepared_solves_equal_the_whole_solve(B, oracle, kind, n, dtype_name):
    """One prepare call, then several solves of different widths with its workspace: each bit for bit what the
    one-call solve gives (same kernels in the same order), and the first one checked against the oracle."""
    import torch
    dtype = getattr(torch, dtype_name)
    announce(f"prepared solve {kind} n={n} {dtype_name}")
    _, F = _factor(oracle, kind, n, 27)
    if dtype_name == "float32":
        F = F.astype(np.float32).astype(np.float64)
    f = to_device(F, dtype)
    whole = B.lu_solve if kind == "lu" else B.cholesky_solve
    ws = (B.lu_solve_prepare if kind == "lu" else B.cholesky_solve_prepare)(f, 130)
    prepared = B.lu_solve_prepared if kind == "lu" else B.cholesky_solve_prepared
    for i, nrhs in enumerate((64, 5, 130, 33)):
        rhs = inputs.uniform_matrix(28, i, n, nrhs)
        if dtype_name == "float32":
            rhs = rhs.astype(np.float32).astype(np.float64)
        b1, b2 = to_device(rhs, dtype), to_device(rhs, dtype)
        whole(f, b1)
        prepared(f, b2, ws)
        x1, x2 = to_host(b1), to_host(b2)
        assert np.array_equal(x1, x2)
        if i == 0:
            want = (oracle.lu_solve if kind == "lu" else oracle.cholesky_solve)(F, rhs)
            assert max_rel_err(x2.astype(np.float64), want) <= (TOL64 if dtype_name == "float64" else TOL32)
    with pytest.raises(Exception):  # more right-hand sides than the workspace was sized for
        prepared(f, to_device(inputs.uniform_matrix(28, 9, n, 200), dtype), ws)


@pytest.mark.parametrize("kind", ["lu", "chol"])
@pytest.mark.parametrize("n,nrhs", [(129, 3), (700, 40), (1025, 20)])
def test_solve_fp32(B, oracle, kind, n, nrhs):
    import torch
    announce(f"solve {kind} n={n} nrhs={nrhs} f32")
    _, F = _factor(oracle, kind, n, 23)
    rhs = inputs.uniform_matrix(24, 3, n, nrhs)
    F32, rhs32 = F.astype(np.float32), rhs.astype(np.float32)
    want = (oracle.lu_solve if kind == "lu" else oracle.cholesky_solve)(F32.astype(np.float64), rhs32.astype(np.float64))
    got = _gpu_solve(B, kind, F32, rhs32, torch.float32)
    assert got.dtype == np.float32
    assert max_rel_err(got.astype(np.float64), want) <= TOL32


@pytest.mark.parametrize("kind", ["lu", "chol"])
def test_solve_with_padded_leading_dimensions(B, oracle, kind):
    """Factor and right-hand sides as views into wider buffers: what lies outside must stay untouched."""
    import torch
    n, nrhs, lda, ldb = 200, 9, 231, 20
    announce(f"solve {kind} n={n} nrhs={nrhs} lda={lda} ldb={ldb}")
    _, F = _factor(oracle, kind, n, 25)
    rhs = inputs.uniform_matrix(26, 3, n, nrhs)
    fbuf = torch.full((n, lda), 7.25, dtype=torch.float64, device="cuda")
    bbuf = torch.full((n, ldb), -3.5, dtype=torch.float64, device="cuda")
    fbuf[:, :n] = to_device(F)
    bbuf[:, :nrhs] = to_device(rhs)
    (B.lu_solve if kind == "lu" else B.cholesky_solve)(fbuf[:, :n], bbuf[:, :nrhs])
    want = (oracle.lu_solve if kind == "lu" else oracle.cholesky_solve)(F, rhs)
    out = to_host(bbuf)
    assert max_rel_err(out[:, :nrhs], want) <= TOL64
    assert np.all(out[:, nrhs:] == -3.5)
    assert np.array_equal(to_host(fbuf)[:, :n], F) and np.all(to_host(fbuf)[:, n:] == 7.25)


def test_cholesky_solve_reads_the_lower_triangle_only(B, oracle):
    n, nrhs = 150, 4
    _, L = _factor(oracle, "chol", n, 27)
    rhs = inputs.uniform_matrix(28, 3, n, nrhs)
    junk = L + np.triu(np.full((n, n), 1e30), 1)
    assert np.array_equal(_gpu_solve(B, "chol", junk, rhs), _gpu_solve(B, "chol", L, rhs))


def test_hand_worked_and_integer_systems(B):
    """The hand-worked fixtures to a few units in the last place (the device multiplies by inverted 16 x 16
    diagonal blocks where the definition divides, and their diagonals 3 and 10 have no exact reciprocal);
    integer systems whose every intermediate value, inverses included, is an exact integer: bit for bit."""
    with open(GOLDEN) as f:
        golden = json.load(f)
    for c in golden["lu_solve"]:
        got = _gpu_solve(B, "lu", np.array(c["LU"], dtype=np.float64), np.array(c["B"], dtype=np.float64))
        np.testing.assert_allclose(got, np.array(c["X"], dtype=np.float64), rtol=8 * EPS64, atol=8 * EPS64, err_msg=c["name"])
    for c in golden["cholesky_solve"]:
        got = _gpu_solve(B, "chol", np.array(c["L"], dtype=np.float64), np.array(c["B"], dtype=np.float64))
        np.testing.assert_allclose(got, np.array(c["X"], dtype=np.float64), rtol=8 * EPS64, atol=8 * EPS64, err_msg=c["name"])
    # bidiagonal unit factors over several blocks and a ragged tail: all inverses are +-1 patterns
    n, nrhs = 300, 20
    Lm = np.eye(n) + np.diag(np.ones(n - 1), -1)
    Um = np.eye(n) - np.diag(np.ones(n - 1), 1)
    X = inputs.integer_matrix(29, 3, n, nrhs, -3, 3)
    announce(f"exact integer solve n={n} nrhs={nrhs}")
    got = _gpu_solve(B, "lu", np.tril(Lm, -1) + Um, Lm @ (Um @ X))
    assert np.array_equal(got, X)
    got = _gpu_solve(B, "chol", Lm, Lm @ (Lm.T @ X))
    assert np.array_equal(got, X)


@pytest.mark.parametrize("kind", ["lu", "chol"])
def test_factor_then_solve_on_the_gpu(B, oracle, kind):
    """End to end: factorisation and solve both on the device, checked by the residual of the system and
    against the oracle's factorisation followed by the oracle's substitutions."""
    n, nrhs = 1500, 33
    announce(f"factor + solve {kind} n={n} nrhs={nrhs}")
    A = inputs.general_dominant_matrix(n, 31) if kind == "lu" else inputs.spd_matrix(n, 31)
    rhs = inputs.uniform_matrix(32, 3, n, nrhs)
    a, b = to_device(A), to_device(rhs)
    if kind == "lu":
        B.lu_factor(a)
        B.lu_solve(a, b)
    else:
        B.cholesky_factor(a)
        B.cholesky_solve(a, b)
    X = to_host(b)
    assert np.abs(A @ X - rhs).max() <= 64 * n * EPS64 * np.abs(A).max() * np.abs(X).max()
    F, info = (oracle.lu if kind == "lu" else oracle.cholesky)(A)
    assert info == 0
    want = (oracle.lu_solve if kind == "lu" else oracle.cholesky_solve)(F, rhs)
    assert max_rel_err(X, want) <= TOL64


def test_cholesky_solve_with_a_condition_number_of_a_thousand(B, oracle):
    """The device multiplies by explicitly inverted 128 x 128 diagonal blocks; their condition enters its
    error.  Gram matrix + 1e-3 I (condition about 1.3e3, against about 2 for the workload recipe's + I):
    the solution still matches the substitution of the oracle, and the system's residual stays small."""
    n, nrhs = 700, 9
    announce(f"solve chol n={n} nrhs={nrhs} shift 1e-3")
    A = inputs.spd_matrix(n, 41)
    A[np.diag_indices(n)] += 1e-3 - 1.0
    F, info = oracle.cholesky(A)
    assert info == 0
    rhs = inputs.uniform_matrix(42, 3, n, nrhs)
    want = oracle.cholesky_solve(F, rhs)
    got = _gpu_solve(B, "chol", F, rhs)
    assert max_rel_err(got, want) <= TOL64
    assert np.abs(A @ got - rhs).max() <= 64 * n * EPS64 * np.abs(A).max() * np.abs(got).max()


def test_n4000_sampled_columns(B, oracle):
    """The benchmark's matrix size: device factor, then the oracle's solve on that factor for a few columns."""
    n, nrhs = 4000, 64
    announce(f"solve lu n={n} nrhs={nrhs}")
    A = inputs.diag_dominant_matrix(n, 33)
    rhs = inputs.uniform_matrix(34, 3, n, nrhs)
    a, b = to_device(A), to_device(rhs)
    B.lu_factor(a)
    F = to_host(a)
    B.lu_solve(a, b)
    X = to_host(b)
    cols = [0, 17, 63]
    want = oracle.lu_solve(F, rhs[:, cols])
    assert max_rel_err(X[:, cols], want) <= TOL64


@pytest.mark.parametrize("m,n,k,tile", [(64, 64, 16, None), (100, 37, 128, None), (300, 129, 77, (32, 32, 16, 4, 16, 16)),
                                        (257, 200, 128, (64, 64, 32, 4, 32, 32))])
def test_transposed_left_operand_product(B, oracle, m, n, k, tile):
    """dla_gemm op 4: C -= A^T * B with A stored k x m."""
    announce(f"gemm op4 m={m} n={n} k={k} tile={tile}")
    a = inputs.uniform_matrix(35, 1, k, m)
    b = inputs.uniform_matrix(35, 2, k, n)
    c = inputs.uniform_matrix(35, 3, m, n)
    ad, bd, cd = to_device(a), to_device(b), to_device(c)
    B.dla_gemm(4, ad, bd, cd, B.GemmParams(*tile) if tile else None)
    want = c - oracle_product(oracle, a.T, b)
    assert max_rel_err(to_host(cd), want) <= 1e-12
    with pytest.raises(RuntimeError):
        B.dla_gemm(4, ad, bd, cd, B.GemmParams(128, 128, 16, 4, 64, 64))  # not instantiated for this macro-tile


def test_empty_systems_are_no_ops(B):
    import torch
    f = torch.empty((0, 0), dtype=torch.float64, device="cuda")
    b = torch.empty((0, 5), dtype=torch.float64, device="cuda")
    B.lu_solve(f, b)
    B.cholesky_solve(f, b)
    f = to_device(np.eye(4))
    b = torch.empty((4, 0), dtype=torch.float64, device="cuda")
    B.lu_solve(f, b)
