"""Pins for the CPU oracle: everything here runs without a GPU.

The oracle is checked against things other than itself: hand-worked fixtures
(re-verified in exact rational arithmetic inside the test), closed forms,
exact-integer matrices with known factors, invariants that tie LU to Cholesky,
brute-force 4-index sums for 3mm, exact rational elimination on tiny inputs,
and library routines on special cases (numpy's Cholesky; a pivoted library LU
on matrices where no row swap occurs; the library's triangular and dense
solvers for the substitutions with the factors).
"""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2309_07235_amd import inputs
from tests.metrics import EPS64, max_rel_err

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_worked.json")


def _frac(m):
    return [[Fraction(v) for v in row] for row in m]


def _fmul(X, Y):
    return [[sum(X[i][k] * Y[k][j] for k in range(len(Y))) for j in range(len(Y[0]))] for i in range(len(X))]


def _tofloat(m):
    return np.array([[float(Fraction(v)) for v in row] for row in m], dtype=np.float64)


@pytest.fixture(scope="module")
def golden():
    with open(GOLDEN) as f:
        return json.load(f)


# ---------------------------------------------------------------- hand-worked fixtures
def test_golden_fixtures_are_exact_factorisations(golden):
    """The stored values themselves: L*U == A, L*L^T == A, E*F == G in exact arithmetic."""
    for c in golden["lu"]:
        A, LU = _frac(c["A"]), _frac(c["LU"])
        n = len(A)
        L = [[LU[i][j] if j < i else Fraction(int(i == j)) for j in range(n)] for i in range(n)]
        U = [[LU[i][j] if j >= i else Fraction(0) for j in range(n)] for i in range(n)]
        assert _fmul(L, U) == A, c["name"]
    for c in golden["cholesky"]:
        A, L = _frac(c["A"]), _frac(c["L"])
        n = len(A)
        assert all(L[i][j] == 0 for i in range(n) for j in range(i + 1, n))
        assert all(L[i][i] > 0 for i in range(n))
        LT = [[L[j][i] for j in range(n)] for i in range(n)]
        assert _fmul(L, LT) == A, c["name"]
    for c in golden["mm3"]:
        A, B, C, D, E, F, G = (_frac(c[k]) for k in "ABCDEFG")
        assert _fmul(A, B) == E and _fmul(C, D) == F and _fmul(E, F) == G, c["name"]


def test_lu_hand_worked(oracle, golden):
    for c in golden["lu"]:
        got, info = oracle.lu(_tofloat(c["A"]))
        assert info == 0
        np.testing.assert_allclose(got, _tofloat(c["LU"]), rtol=4 * EPS64, atol=0, err_msg=c["name"])


def test_cholesky_hand_worked(oracle, golden):
    for c in golden["cholesky"]:
        got, info = oracle.cholesky(_tofloat(c["A"]))
        assert info == 0
        assert np.array_equal(got, _tofloat(c["L"])), c["name"]  # integer data: exact


def test_mm3_hand_worked(oracle, golden):
    for c in golden["mm3"]:
        G, E, F = oracle.mm3(*(_tofloat(c[k]) for k in "ABCD"), return_intermediates=True)
        assert np.array_equal(E, _tofloat(c["E"])), c["name"]
        assert np.array_equal(F, _tofloat(c["F"])), c["name"]
        assert np.array_equal(G, _tofloat(c["G"])), c["name"]


# ---------------------------------------------------------------- identity / diagonal
def test_identity_and_diagonal(oracle):
    n = 7
    I = np.eye(n)
    assert np.array_equal(oracle.lu(I)[0], I)
    assert np.array_equal(oracle.cholesky(I)[0], I)
    d = np.array([4.0, 9.0, 0.25, 16.0, 1.0, 2.25, 100.0])
    assert np.array_equal(oracle.lu(np.diag(d))[0], np.diag(d))
    assert np.array_equal(oracle.cholesky(np.diag(d))[0], np.diag(np.sqrt(d)))
    A = inputs.uniform_matrix(5, 0, n, n)
    D = inputs.uniform_matrix(5, 1, n, 4)
    G = oracle.mm3(A, I, I, D)
    ref = np.array([[math.fsum(A[i, k] * D[k, j] for k in range(n)) for j in range(4)] for i in range(n)])
    np.testing.assert_allclose(G, ref, rtol=0, atol=8 * EPS64 * n)


# ---------------------------------------------------------------- exact integer matrices
@pytest.mark.parametrize("n", [1, 2, 17, 64, 200])
def test_min_index_matrix_has_all_ones_factors(oracle, n):
    """A[i][j] = min(i, j) + 1: L = ones lower (both factorisations), U = ones upper; all exact."""
    A = inputs.min_index_matrix(n)
    lu, info = oracle.lu(A)
    assert info == 0 and np.array_equal(lu, np.ones((n, n)))
    L, info = oracle.cholesky(A)
    assert info == 0 and np.array_equal(L, np.tril(np.ones((n, n))))


@pytest.mark.parametrize("n", [2, 5, 12, 16])
def test_symmetric_pascal_matrix(oracle, n):
    """S[i][j] = C(i+j, i): Cholesky factor L[i][j] = C(i, j); LU = (L, L^T). Exact integers."""
    S = np.array([[math.comb(i + j, i) for j in range(n)] for i in range(n)], dtype=np.float64)
    Lref = np.array([[math.comb(i, j) for j in range(n)] for i in range(n)], dtype=np.float64)
    L, info = oracle.cholesky(S)
    assert info == 0 and np.array_equal(L, Lref)
    lu, info = oracle.lu(S)
    assert info == 0
    assert np.array_equal(np.tril(lu, -1), np.tril(Lref, -1))
    assert np.array_equal(np.triu(lu), Lref.T)


def test_mm3_integer_inputs_match_int64_arithmetic(oracle):
    """Integer entries in {-3..3}: every partial sum is an exact integer, compare with int64 matmul."""
    dims = dict(ni=23, nk=31, nj=17, nm=29, nl=13)
    A, B, C, D = inputs.mm3_integer_operands(7, **dims)
    G, E, F = oracle.mm3(A, B, C, D, return_intermediates=True)
    Ai, Bi, Ci, Di = (x.astype(np.int64) for x in (A, B, C, D))
    assert np.array_equal(E, (Ai @ Bi).astype(np.float64))
    assert np.array_equal(F, (Ci @ Di).astype(np.float64))
    assert np.array_equal(G, ((Ai @ Bi) @ (Ci @ Di)).astype(np.float64))


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("n", [3, 10, 50])
def test_tridiagonal_closed_form(oracle, n):
    """tridiag(-1, 2, -1): u_ii = (i+1)/i, l_{i+1,i} = -i/(i+1) (1-based); Cholesky the square roots."""
    A = 2 * np.eye(n) - np.eye(n, k=1) - np.eye(n, k=-1)
    lu, info = oracle.lu(A)
    assert info == 0
    for i in range(1, n + 1):
        assert lu[i - 1, i - 1] == pytest.approx((i + 1) / i, rel=1e-14)
        if i < n:
            assert lu[i, i - 1] == pytest.approx(-i / (i + 1), rel=1e-14)
            assert lu[i - 1, i] == -1.0
    band = np.abs(np.subtract.outer(np.arange(n), np.arange(n))) > 1
    assert np.all(lu[band] == 0.0)
    L, info = oracle.cholesky(A)
    assert info == 0
    for i in range(1, n + 1):
        assert L[i - 1, i - 1] == pytest.approx(math.sqrt((i + 1) / i), rel=1e-14)
        if i < n:
            assert L[i, i - 1] == pytest.approx(-math.sqrt(i / (i + 1)), rel=1e-14)
    assert np.all(L[band] == 0.0)


# ---------------------------------------------------------------- exact rational brute force
def _rational_lu(A):
    """Unique unit-lower/upper factors from the defining equations, solved entry by entry."""
    n = len(A)
    L = [[Fraction(int(i == j)) for j in range(n)] for i in range(n)]
    U = [[Fraction(0)] * n for _ in range(n)]
    for s in range(n):
        for j in range(s, n):  # row s of U from  A[s][j] = sum_k L[s][k] U[k][j]
            U[s][j] = A[s][j] - sum(L[s][k] * U[k][j] for k in range(s))
        for i in range(s + 1, n):  # column s of L from  A[i][s] = sum_k L[i][k] U[k][s]
            L[i][s] = (A[i][s] - sum(L[i][k] * U[k][s] for k in range(s))) / U[s][s]
    return L, U


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_lu_against_exact_rational_solution(oracle, seed):
    """Non-symmetric integer matrix: compare with the exact factors (Crout-order rational solve)."""
    n = 6
    Ai = inputs.integer_matrix(seed, 3, n, n, -4, 4) + 9 * np.eye(n)
    L, U = _rational_lu(_frac(Ai.astype(int).tolist()))
    want = np.array([[float(L[i][j]) if j < i else float(U[i][j]) for j in range(n)] for i in range(n)])
    got, info = oracle.lu(Ai)
    assert info == 0
    np.testing.assert_allclose(got, want, rtol=64 * EPS64, atol=64 * EPS64)


def test_lu_is_not_symmetric_in_its_argument(oracle):
    """A transposed operand anywhere in the elimination would make LU(A^T) == LU(A)^T-like mistakes pass; it must not."""
    A = np.array([[4.0, 1.0, 2.0], [8.0, 5.0, 1.0], [12.0, 9.0, 10.0]])
    got, _ = oracle.lu(A)
    # exact: L = [[1,0,0],[2,1,0],[3,2,1]], U = [[4,1,2],[0,3,-3],[0,0,10]]
    assert np.array_equal(got, np.array([[4.0, 1.0, 2.0], [2.0, 3.0, -3.0], [3.0, 2.0, 10.0]]))


# ---------------------------------------------------------------- invariants
@pytest.mark.parametrize("n", [5, 40, 129])
def test_lu_and_cholesky_are_tied_for_spd_input(oracle, n):
    """For SPD A with Cholesky factor C: L_lu = C diag(C)^-1 and U = diag(C) C^T."""
    A = inputs.spd_matrix(n, 11)
    C, info = oracle.cholesky(A)
    assert info == 0
    lu, info = oracle.lu(A)
    assert info == 0
    d = np.diag(C)
    Lref = np.tril(C / d[None, :], -1)
    Uref = np.triu(d[:, None] * C.T)
    assert max_rel_err(np.tril(lu, -1) + Uref * 0, Lref) < 1e-12
    assert max_rel_err(np.triu(lu), Uref) < 1e-12


@pytest.mark.parametrize("n", [1, 33, 300])
def test_reconstruction_and_structure(oracle, n):
    A = inputs.diag_dominant_matrix(n, 3)
    lu, info = oracle.lu(A)
    assert info == 0
    L = np.tril(lu, -1) + np.eye(n)
    U = np.triu(lu)
    assert np.linalg.norm(A - L @ U) <= 10 * n * EPS64 * np.linalg.norm(A)
    assert oracle.lu_residual(A, lu) <= 10 * n * EPS64

    S = inputs.spd_matrix(n, 2)
    C, info = oracle.cholesky(S)
    assert info == 0
    assert np.all(np.triu(C, 1) == 0.0) and np.all(np.diag(C) > 0)
    assert np.linalg.norm(S - C @ C.T) <= 10 * n * EPS64 * np.linalg.norm(S)
    assert oracle.cholesky_residual(S, C) <= 10 * n * EPS64


def test_residual_helpers_detect_a_wrong_factor(oracle):
    """The residual routines themselves: exact value on a case worked by hand, and they see a planted error."""
    A = np.array([[4.0, 2.0], [2.0, 5.0]])
    L = np.array([[2.0, 0.0], [1.0, 2.0]])
    assert oracle.cholesky_residual(A, L) == 0.0
    Lbad = L.copy()
    Lbad[1, 0] = 1.5  # L L^T = [[4,3],[3,6.25]]: residual entries (2,1)->-1 twice, (2,2)->-1.25
    want = math.sqrt((2 * 1.0 + 1.25 ** 2) / (16 + 2 * 4 + 25))
    assert oracle.cholesky_residual(A, Lbad) == pytest.approx(want, rel=1e-15)
    lu = np.array([[4.0, 2.0], [0.5, 4.0]])
    assert oracle.lu_residual(A, lu) == 0.0
    lub = lu.copy()
    lub[0, 1] = 3.0  # L U = [[4,3],[2,5.5]]
    assert oracle.lu_residual(A, lub) == pytest.approx(math.sqrt((1 + 0.25) / 49), rel=1e-15)


def test_apply_helpers(oracle):
    n = 57
    A = inputs.general_dominant_matrix(n, 9)
    lu, _ = oracle.lu(A)
    x = inputs.uniform_matrix(9, 5, n, 1).ravel()
    L = np.tril(lu, -1) + np.eye(n)
    U = np.triu(lu)
    np.testing.assert_allclose(oracle.lu_apply(lu, x), L @ (U @ x), rtol=1e-13)
    np.testing.assert_allclose(oracle.matvec(A, x), A @ x, rtol=1e-13, atol=1e-13)
    S = inputs.spd_matrix(n, 4)
    C, _ = oracle.cholesky(S)
    np.testing.assert_allclose(oracle.cholesky_apply(C, x), C @ (C.T @ x), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(oracle.symv_lower(np.tril(S), x), S @ x, rtol=1e-12, atol=1e-13)


def test_cholesky_reads_lower_triangle_only(oracle):
    S = inputs.spd_matrix(20, 8)
    junk = np.tril(S) + np.triu(np.full((20, 20), 1e30), 1)
    assert np.array_equal(oracle.cholesky(junk)[0], oracle.cholesky(S)[0])


# ---------------------------------------------------------------- 3mm brute force / associativity
@pytest.mark.parametrize("dims", [(2, 3, 4, 5, 6), (6, 5, 4, 3, 2), (1, 1, 1, 1, 1), (4, 6, 3, 6, 5)])
def test_mm3_brute_force_four_index_sum(oracle, dims):
    ni, nk, nj, nm, nl = dims
    A, B, C, D = inputs.mm3_operands(21, ni, nk, nj, nm, nl)
    G = oracle.mm3(A, B, C, D)
    want = np.zeros((ni, nl))
    for i in range(ni):
        for j in range(nl):
            want[i, j] = math.fsum(A[i, k] * B[k, m] * C[m, l] * D[l, j]
                                   for k in range(nk) for m in range(nj) for l in range(nm))
    np.testing.assert_allclose(G, want, rtol=0, atol=1e-13)
    # associativity: ((A B) C) D and A (B (C D)) agree with (A B)(C D)
    np.testing.assert_allclose(((A @ B) @ C) @ D, G, rtol=0, atol=1e-13)
    np.testing.assert_allclose(A @ (B @ (C @ D)), G, rtol=0, atol=1e-13)


def test_mm3_integer_associativity_is_exact(oracle):
    A, B, C, D = inputs.mm3_integer_operands(3, 5, 6, 4, 3, 6)
    G = oracle.mm3(A, B, C, D)
    want = np.zeros_like(G)
    for i in range(5):
        for j in range(6):
            want[i, j] = sum(int(A[i, k]) * int(B[k, m]) * int(C[m, l]) * int(D[l, j])
                             for k in range(6) for m in range(4) for l in range(3))
    assert np.array_equal(G, want)


def test_mm3_rejects_mismatched_inner_dimensions(oracle):
    with pytest.raises(ValueError):
        oracle.mm3(np.zeros((2, 3)), np.zeros((4, 2)), np.zeros((2, 2)), np.zeros((2, 2)))


# ---------------------------------------------------------------- library witnesses
@pytest.mark.parametrize("n", [64, 257])
def test_cholesky_matches_numpy_library(oracle, n):
    S = inputs.spd_matrix(n, 2)
    L, info = oracle.cholesky(S)
    assert info == 0
    assert max_rel_err(L, np.linalg.cholesky(S)) < 1e-12


def test_lu_matches_pivoted_library_when_no_swap_occurs(oracle):
    scipy_linalg = pytest.importorskip("scipy.linalg")
    n = 200
    A = inputs.general_dominant_matrix(n, 3)
    lu_lib, piv = scipy_linalg.lu_factor(A)
    assert np.array_equal(piv, np.arange(n))  # dominance: partial pivoting never swaps
    got, info = oracle.lu(A)
    assert info == 0
    assert max_rel_err(got, lu_lib) < 1e-12


# ---------------------------------------------------------------- breakdown reporting
def test_zero_pivot_and_indefinite_input_are_reported(oracle):
    A = np.array([[1.0, 2.0, 3.0], [2.0, 4.0, 1.0], [1.0, 1.0, 1.0]])  # second pivot 4 - 2*2 = 0
    assert oracle.lu(A)[1] == 2
    assert oracle.lu(np.zeros((3, 3)))[1] == 1
    S = np.array([[4.0, 2.0, 0.0], [2.0, 1.0, 0.0], [0.0, 0.0, 1.0]])  # second pivot 1 - 1 = 0
    assert oracle.cholesky(S)[1] == 2
    assert oracle.cholesky(-np.eye(3))[1] == 1
    assert oracle.cholesky(np.diag([1.0, float("nan"), 1.0]))[1] == 2


# ---------------------------------------------------------------- generators
def test_generators_are_counter_based_and_seeded():
    a = inputs.uniform_matrix(4, 10, 7, 9)
    b = inputs.uniform_matrix(4, 10, 7, 9)
    assert np.array_equal(a, b)
    assert not np.array_equal(a, inputs.uniform_matrix(5, 10, 7, 9))
    assert not np.array_equal(a, inputs.uniform_matrix(4, 11, 7, 9))
    flat = inputs.uniform_matrix(4, 10, 1, 63)
    assert np.array_equal(a.ravel(), flat.ravel())  # element depends on the flat index only
    big = inputs.uniform_matrix(1, 0, 300, 300)
    assert -1.0 <= big.min() and big.max() < 1.0
    assert abs(big.mean()) < 0.02 and abs(big.var() - 1.0 / 3.0) < 0.02
    S = inputs.spd_matrix(50, 2)
    assert np.array_equal(S, S.T)
    w = np.linalg.eigvalsh(S)
    assert w.min() >= 1.0 - 1e-12
    Ai = inputs.integer_matrix(3, 0, 40, 40)
    assert np.array_equal(Ai, np.round(Ai)) and Ai.min() >= -3 and Ai.max() <= 3
    assert len(np.unique(Ai)) == 7


# ---------------------------------------------------------------- solving with the factors
def test_solve_fixtures_are_exact_and_reproduced(oracle, golden):
    """Hand-worked systems: the stored X satisfies (L*U)*X == B resp. (L*L^T)*X == B exactly, and the
    oracle returns it bit for bit (all intermediate values are small integers)."""
    for c in golden["lu_solve"]:
        LU, B, X = _frac(c["LU"]), _frac(c["B"]), _frac(c["X"])
        n = len(LU)
        L = [[LU[i][j] if j < i else Fraction(int(i == j)) for j in range(n)] for i in range(n)]
        U = [[LU[i][j] if j >= i else Fraction(0) for j in range(n)] for i in range(n)]
        assert _fmul(_fmul(L, U), X) == B, c["name"]
        assert np.array_equal(oracle.lu_solve(_tofloat(c["LU"]), _tofloat(c["B"])), _tofloat(c["X"])), c["name"]
    for c in golden["cholesky_solve"]:
        L, B, X = _frac(c["L"]), _frac(c["B"]), _frac(c["X"])
        n = len(L)
        LT = [[L[j][i] for j in range(n)] for i in range(n)]
        assert _fmul(_fmul(L, LT), X) == B, c["name"]
        assert np.array_equal(oracle.cholesky_solve(_tofloat(c["L"]), _tofloat(c["B"])), _tofloat(c["X"])), c["name"]


def test_lu_solve_ignores_the_stored_diagonal_in_the_forward_pass(oracle):
    """The diagonal of an in-place LU result belongs to U: dividing by it in the forward pass, or using L's
    implied ones in the backward pass, changes the 3x3 fixture's answer."""
    LU = np.array([[4.0, 1.0, 2.0], [2.0, 3.0, -3.0], [3.0, 2.0, 10.0]])
    b = np.array([12.0, 21.0, 60.0])
    x = oracle.lu_solve(LU, b)
    assert np.array_equal(x, [1.0, 2.0, 3.0])
    L = np.tril(LU, -1) + np.eye(3)
    U = np.triu(LU)
    wrong_forward = np.linalg.solve(U, np.linalg.solve(np.tril(LU), b))          # divided by U's diagonal
    wrong_backward = np.linalg.solve(np.triu(LU, 1) + np.eye(3), np.linalg.solve(L, b))  # unit U
    assert not np.allclose(x, wrong_forward) and not np.allclose(x, wrong_backward)


def test_cholesky_solve_uses_the_transpose_in_the_backward_pass(oracle):
    L = np.array([[2.0, 0.0, 0.0], [1.0, 3.0, 0.0], [-1.0, 2.0, 1.0]])
    b = np.array([6.0, 27.0, 14.0])
    x = oracle.cholesky_solve(L, b)
    assert np.array_equal(x, [1.0, 2.0, 1.0])
    forward_twice = np.linalg.solve(L, np.linalg.solve(L, b))
    assert not np.allclose(x, forward_twice)
    # only the lower triangle is read
    junk = L + np.triu(np.full((3, 3), 7.0), 1)
    assert np.array_equal(oracle.cholesky_solve(junk, b), x)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_lu_solve_against_exact_rational_solution(oracle, seed):
    n, nrhs = 6, 3
    Ai = inputs.integer_matrix(seed, 3, n, n, -4, 4) + 9 * np.eye(n)
    Bi = inputs.integer_matrix(seed, 4, n, nrhs, -5, 5)
    A = _frac(Ai.astype(int).tolist())
    L, U = _rational_lu(A)
    # exact solution by substitution in rationals
    X = [[Fraction(0)] * nrhs for _ in range(n)]
    for c in range(nrhs):
        y = [Fraction(0)] * n
        for i in range(n):
            y[i] = Fraction(int(Bi[i, c])) - sum(L[i][j] * y[j] for j in range(i))
        for i in reversed(range(n)):
            X[i][c] = (y[i] - sum(U[i][j] * X[j][c] for j in range(i + 1, n))) / U[i][i]
    assert _fmul(A, X) == _frac(Bi.astype(int).tolist())
    lu, info = oracle.lu(Ai)
    assert info == 0
    got = oracle.lu_solve(lu, Bi)
    np.testing.assert_allclose(got, _tofloat(X), rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("n,nrhs", [(1, 1), (40, 1), (129, 7)])
def test_solves_match_library_routines(oracle, n, nrhs):
    scipy_linalg = pytest.importorskip("scipy.linalg")
    A = inputs.general_dominant_matrix(n, 6)
    S = inputs.spd_matrix(n, 7)
    B = inputs.uniform_matrix(8, 1, n, nrhs)
    lu, info = oracle.lu(A)
    assert info == 0
    X = oracle.lu_solve(lu, B)
    assert max_rel_err(X, np.linalg.solve(A, B)) < 1e-11
    # the two substitutions one at a time, with the library's triangular solver on the same factors
    Y = scipy_linalg.solve_triangular(lu, B, lower=True, unit_diagonal=True)
    assert max_rel_err(X, scipy_linalg.solve_triangular(lu, Y, lower=False)) < 1e-12
    Lc, info = oracle.cholesky(S)
    assert info == 0
    Xc = oracle.cholesky_solve(Lc, B)
    assert max_rel_err(Xc, scipy_linalg.cho_solve((Lc, True), B)) < 1e-12
    assert max_rel_err(Xc, np.linalg.solve(S, B)) < 1e-10


def test_solve_invariants(oracle):
    n, nrhs = 50, 4
    A = inputs.general_dominant_matrix(n, 9)
    B = inputs.uniform_matrix(9, 2, n, nrhs)
    lu, _ = oracle.lu(A)
    X = oracle.lu_solve(lu, B)
    assert np.abs(A @ X - B).max() <= 64 * n * EPS64 * np.abs(A).max() * np.abs(X).max()
    # columns are independent systems: solving them one at a time gives the same bits
    for c in range(nrhs):
        assert np.array_equal(oracle.lu_solve(lu, B[:, c]), X[:, c])
    # identity and diagonal factors
    assert np.array_equal(oracle.lu_solve(np.eye(n), B), B)
    d = np.arange(1.0, n + 1.0)
    assert np.array_equal(oracle.lu_solve(np.diag(d), B), B / d[:, None])
    np.testing.assert_allclose(oracle.cholesky_solve(np.diag(d), B), B / (d * d)[:, None], rtol=4 * EPS64)
    with pytest.raises(ValueError):
        oracle.lu_solve(lu, B[:-1])
