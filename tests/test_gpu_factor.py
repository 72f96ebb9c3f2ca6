"""GPU parity of lu_factor and cholesky_factor against the CPU oracle."""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2309_07235_amd import inputs
from tests.gpu_util import announce, oracle_product, to_device, to_host
from tests.metrics import EPS32, EPS64, cholesky_rel_err, lu_rel_err, max_rel_err

pytestmark = pytest.mark.gpu

TOL64 = 1e-9   # max relative error; L, strict upper U and the diagonal each floored at their own RMS (tests/metrics.py)
TOL32 = 1e-4
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_worked.json")


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2309_07235_amd import binding
    return binding


def _fparams(B, nb=0, lookahead=-1, tile=None, defer_min_rows=0):
    t = B.GemmParams(*(tile or (0, 0)), *([0] * (6 - len(tile or (0, 0)))))
    return B.FactorParams(nb, lookahead, t, defer_min_rows)


def _gpu_lu(B, A, params=None, dtype=None, want_info=True):
    import torch
    a = to_device(A, dtype)
    info = torch.full((1,), -99, dtype=torch.int32, device="cuda") if want_info else None
    B.lu_factor(a, params, info=info)
    out = to_host(a)
    return out, (int(info.item()) if want_info else None)


def _gpu_chol(B, A, params=None, dtype=None, want_info=True):
    import torch
    a = to_device(A, dtype)
    info = torch.full((1,), -99, dtype=torch.int32, device="cuda") if want_info else None
    B.cholesky_factor(a, params, info=info)
    out = to_host(a)
    return out, (int(info.item()) if want_info else None)


def _check_lu(oracle, got, A, n, tol=TOL64, eps=EPS64):
    want, info = oracle.lu(A)
    assert info == 0
    assert lu_rel_err(got, want) <= tol
    assert oracle.lu_residual(A, got) <= 10 * max(n, 1) * eps


def _check_chol(oracle, got, A, n, tol=TOL64, eps=EPS64):
    want, info = oracle.cholesky(A)
    assert info == 0
    low = np.tril(np.ones((n, n), dtype=bool))
    assert cholesky_rel_err(got, want) <= tol
    assert np.all(got[~low] == 0.0), "strict upper triangle must be exactly zero"
    assert oracle.cholesky_residual(A, got) <= 10 * max(n, 1) * eps


# ------------------------------------------------------------------ small and ragged sizes
@pytest.mark.parametrize("n", [1, 2, 3, 15, 16, 17, 31, 100, 128, 129, 200, 333])
@pytest.mark.parametrize("nb", [16, 48, 128])
def test_lu_small_sizes(B, oracle, n, nb):
    announce(f"lu n={n} nb={nb}")
    A = inputs.general_dominant_matrix(n, 100 + n)
    got, info = _gpu_lu(B, A, _fparams(B, nb))
    assert info == 0
    _check_lu(oracle, got, A, n)


@pytest.mark.parametrize("n", [1, 2, 3, 15, 16, 17, 31, 100, 128, 129, 200, 333])
@pytest.mark.parametrize("nb", [16, 48, 128])
def test_cholesky_small_sizes(B, oracle, n, nb):
    announce(f"cholesky n={n} nb={nb}")
    A = inputs.spd_matrix(n, 200 + n)
    got, info = _gpu_chol(B, A, _fparams(B, nb))
    assert info == 0
    _check_chol(oracle, got, A, n)


def test_hand_worked_fixtures_on_gpu(B):
    announce("hand-worked fixtures")
    with open(GOLDEN) as f:
        g = json.load(f)
    tofloat = lambda m: np.array([[float(Fraction(v)) for v in r] for r in m])
    for c in g["lu"]:
        got, info = _gpu_lu(B, tofloat(c["A"]))
        assert info == 0
        np.testing.assert_allclose(got, tofloat(c["LU"]), rtol=8 * EPS64, atol=0, err_msg=c["name"])
    for c in g["cholesky"]:
        got, info = _gpu_chol(B, tofloat(c["A"]))
        assert info == 0
        np.testing.assert_allclose(got, tofloat(c["L"]), rtol=8 * EPS64, atol=0, err_msg=c["name"])


# ------------------------------------------------------------------ exact integer matrices, bit for bit
@pytest.mark.parametrize("n,nb", [(517, 128), (517, 48), (1000, 64), (2048, 128)])
def test_min_index_matrix_is_bit_exact(B, oracle, n, nb):
    """A[i][j] = min(i, j) + 1 has all-ones factors; every intermediate is a small integer."""
    announce(f"min-index exact n={n} nb={nb}")
    A = inputs.min_index_matrix(n)
    got, info = _gpu_lu(B, A, _fparams(B, nb))
    assert info == 0 and np.array_equal(got, np.ones((n, n)))
    got, info = _gpu_chol(B, A, _fparams(B, nb))
    assert info == 0 and np.array_equal(got, np.tril(np.ones((n, n))))
    if n <= 600:  # and the oracle agrees with the closed form at this size
        assert np.array_equal(oracle.lu(A)[0], np.ones((n, n)))


def test_pascal_matrix_is_bit_exact(B, oracle):
    announce("pascal 14")
    n = 14
    S = np.array([[math.comb(i + j, i) for j in range(n)] for i in range(n)], dtype=np.float64)
    got, info = _gpu_chol(B, S)
    want, _ = oracle.cholesky(S)
    assert info == 0 and np.array_equal(got, want)
    got, info = _gpu_lu(B, S)
    want, _ = oracle.lu(S)
    assert info == 0 and np.array_equal(got, want)


# ------------------------------------------------------------------ the named configurations
def test_cholesky_n1024_nb64(B, oracle):
    announce("cholesky N=1024 nb=64")
    A = inputs.spd_matrix(1024, 2)
    got, info = _gpu_chol(B, A, _fparams(B, 64))
    assert info == 0
    _check_chol(oracle, got, A, 1024)


def test_cholesky_n2000_large_dataset(B, oracle):
    announce("cholesky N=2000 (the paper's large dataset), default schedule")
    A = inputs.spd_matrix(2000, 3)
    got, info = _gpu_chol(B, A)
    assert info == 0
    _check_chol(oracle, got, A, 2000)


def test_lu_n2000_nb128(B, oracle):
    announce("lu N=2000 nb=128 (last block 80)")
    A = inputs.diag_dominant_matrix(2000, 3)
    got, info = _gpu_lu(B, A, _fparams(B, 128))
    assert info == 0
    _check_lu(oracle, got, A, 2000)


@pytest.mark.parametrize("lookahead", [0, 1, 2])
def test_n4000_both(B, oracle, lookahead):
    """The size the headline metric is quoted on, in the launch configuration the benchmark uses."""
    announce(f"lu + cholesky N=4000 lookahead={lookahead}")
    A = inputs.diag_dominant_matrix(4000, 5)
    got, info = _gpu_lu(B, A, _fparams(B, 0, lookahead))
    assert info == 0
    _check_lu(oracle, got, A, 4000)
    S = inputs.spd_matrix(4000, 5)
    got, info = _gpu_chol(B, S, _fparams(B, 0, lookahead))
    assert info == 0
    _check_chol(oracle, got, S, 4000)


def test_n8192_properties(B, oracle):
    """N=8192: exact all-ones factors of the min-index matrix, and a randomised O(N^2)
    reconstruction check of the seeded random inputs with the oracle's matrix-vector routines."""
    n = 8192
    announce("N=8192 min-index exact")
    A = inputs.min_index_matrix(n)
    got, info = _gpu_lu(B, A)
    assert info == 0 and np.array_equal(got, np.ones((n, n)))
    got, info = _gpu_chol(B, A)
    assert info == 0 and np.array_equal(got, np.tril(np.ones((n, n))))
    del A, got
    announce("N=8192 LU reconstruction")
    A = inputs.diag_dominant_matrix(n, 6)
    lu, info = _gpu_lu(B, A)
    assert info == 0
    for t in range(4):
        x = inputs.uniform_matrix(6, 50 + t, n, 1).ravel()
        y0 = oracle.matvec(A, x)
        y1 = oracle.lu_apply(lu, x)
        assert np.linalg.norm(y0 - y1) <= 10 * n * EPS64 * np.linalg.norm(y0)
    announce("N=8192 LU sampled rows against the oracle's full factorisation")
    want, _ = oracle.lu(A)
    assert lu_rel_err(lu, want) <= TOL64
    del want, lu
    announce("N=8192 Cholesky reconstruction")
    A[np.diag_indices(n)] += 1.0 - float(n)  # same Gram matrix, +I instead of +N*I: the SPD generator
    L, info = _gpu_chol(B, A)
    assert info == 0
    assert np.all(np.triu(L, 1) == 0.0)
    for t in range(4):
        x = inputs.uniform_matrix(6, 60 + t, n, 1).ravel()
        y0 = oracle.symv_lower(A, x)
        y1 = oracle.cholesky_apply(L, x)
        assert np.linalg.norm(y0 - y1) <= 10 * n * EPS64 * np.linalg.norm(y0)
    announce("N=8192 Cholesky against the oracle's full factorisation")
    want, _ = oracle.cholesky(A)
    assert cholesky_rel_err(L, want) <= TOL64


@pytest.mark.parametrize("kind,n", [("lu", 5000), ("lu", 3500), ("chol", 6100), ("chol", 4700)])
def test_sizes_around_the_two_level_bulk_update(B, oracle, kind, n):
    """Large trailing matrices take their bulk updates two panels at a time; these sizes start and end that
    regime at different step parities and have a ragged last block.  Element by element against the oracle."""
    announce(f"two-level {kind} n={n}")
    if kind == "lu":
        A = inputs.diag_dominant_matrix(n, 81)
        got, info = _gpu_lu(B, A)
        assert info == 0
        _check_lu(oracle, got, A, n)
    else:
        A = inputs.spd_matrix(n, 82)
        got, info = _gpu_chol(B, A)
        assert info == 0
        _check_chol(oracle, got, A, n)


@pytest.mark.parametrize("nb", [160, 192, 224, 256])
@pytest.mark.parametrize("n", [700, 2100])
def test_two_level_block_sizes(B, oracle, nb, n):
    """Block sizes above 128: panels of two sub-panels, bulk updates of depth nb.  Element by element against the
    oracle in fp64, and in fp32 against the fp64 oracle on the fp32-rounded input; sizes with a ragged last block,
    both look-ahead modes of the pipeline."""
    import torch
    announce(f"two-level nb={nb} n={n}")
    A = inputs.general_dominant_matrix(n, 90 + nb)
    S = inputs.spd_matrix(n, 91 + nb)
    for la in (1, 2):
        got, info = _gpu_lu(B, A, _fparams(B, nb, la))
        assert info == 0
        _check_lu(oracle, got, A, n)
        got, info = _gpu_chol(B, S, _fparams(B, nb, la))
        assert info == 0
        _check_chol(oracle, got, S, n)
    A32, S32 = A.astype(np.float32), S.astype(np.float32)
    got, info = _gpu_lu(B, A32, _fparams(B, nb), dtype=torch.float32)
    assert info == 0 and got.dtype == np.float32
    _check_lu(oracle, got.astype(np.float64), A32.astype(np.float64), n, TOL32, EPS32)
    got, info = _gpu_chol(B, S32, _fparams(B, nb), dtype=torch.float32)
    assert info == 0
    _check_chol(oracle, got.astype(np.float64), S32.astype(np.float64), n, TOL32, EPS32)


@pytest.mark.parametrize("defer", [-1, 1, 1024])
def test_deferral_threshold_is_a_parameter(B, oracle, defer):
    """nb = 128 with the two-level bulk update never, always, and from 1024 rows on: same factors to rounding;
    the number of bulk launches shows which schedule ran."""
    announce(f"defer_min_rows={defer}")
    n = 2500
    A = inputs.diag_dominant_matrix(n, 95)
    S = inputs.spd_matrix(n, 96)
    B.profile_enable(True)
    got, info = _gpu_lu(B, A, _fparams(B, 128, 1, None, defer))
    B.profile_enable(False)
    _, launches, _ = B.profile_read(B.PHASE_UPDATE)
    for ph in (B.PHASE_GEMM, B.PHASE_DIAG, B.PHASE_TRSM):
        B.profile_read(ph)
    assert info == 0
    _check_lu(oracle, got, A, n)
    steps = (n + 127) // 128 - 1
    if defer == -1:
        assert launches >= steps - 2
    elif defer == 1:
        assert launches <= steps // 2 + 3
    got, info = _gpu_chol(B, S, _fparams(B, 128, 1, None, defer))
    assert info == 0
    _check_chol(oracle, got, S, n)


def test_min_index_matrix_is_bit_exact_with_two_levels(B):
    announce("min-index exact, nb=256 and nb=192, n=3000")
    n = 3000
    A = inputs.min_index_matrix(n)
    for nb in (256, 192):
        got, info = _gpu_lu(B, A, _fparams(B, nb))
        assert info == 0 and np.array_equal(got, np.ones((n, n)))
        got, info = _gpu_chol(B, A, _fparams(B, nb))
        assert info == 0 and np.array_equal(got, np.tril(np.ones((n, n))))


# ------------------------------------------------------------------ schedules
@pytest.mark.parametrize("tile", [(16, 16), (64, 64), (128, 128), (128, 64), (256, 128)])
def test_update_schedules(B, oracle, tile):
    announce(f"factor update tile {tile}")
    n = 700
    A = inputs.general_dominant_matrix(n, 31)
    got, info = _gpu_lu(B, A, _fparams(B, 64, 0, tile))
    assert info == 0
    _check_lu(oracle, got, A, n)
    if tile[0] == tile[1]:
        S = inputs.spd_matrix(n, 32)
        got, info = _gpu_chol(B, S, _fparams(B, 64, 0, tile))
        assert info == 0
        _check_chol(oracle, got, S, n)


def test_rectangular_tile_is_refused_for_cholesky(B):
    import torch
    a = to_device(inputs.spd_matrix(64, 1))
    with pytest.raises(B.DlaError) as e:
        B.cholesky_factor(a, _fparams(B, 64, 0, (128, 64)))
    assert e.value.code == B.DLA_ERR_UNSUPPORTED_PARAMS


# ------------------------------------------------------------------ breakdown reporting
def test_zero_pivot_index_matches_oracle(B, oracle):
    announce("lu zero pivot")
    n, k = 300, 201
    A = inputs.general_dominant_matrix(n, 40)
    A[k, :] = A[k - 1, :]  # rows k-1 and k equal: pivot k (0-based) becomes exactly zero
    A[:, k] = A[:, k - 1]
    A[k, k] = A[k - 1, k - 1]
    want_info = oracle.lu(A)[1]
    assert want_info == k + 1
    _, info = _gpu_lu(B, A, _fparams(B, 64))
    assert info == want_info
    _, info = _gpu_lu(B, np.zeros((5, 5)))
    assert info == 1


def test_indefinite_matrix_index_matches_oracle(B, oracle):
    announce("cholesky non-positive pivot")
    n, k = 260, 150
    S = inputs.spd_matrix(n, 41)
    S[k, k] = -5.0
    want_info = oracle.cholesky(S)[1]
    assert want_info == k + 1
    _, info = _gpu_chol(B, S, _fparams(B, 64))
    assert info == want_info
    _, info = _gpu_chol(B, -np.eye(3))
    assert info == 1


def test_info_pointer_is_optional(B, oracle):
    """Without an info pointer a wait that gives up could not be reported, so the pipeline (n above two
    blocks) is then ordered by stream events even when in-kernel hand-over is asked for."""
    announce("info=NULL")
    A = inputs.general_dominant_matrix(90, 42)
    got, _ = _gpu_lu(B, A, want_info=False)
    _check_lu(oracle, got, A, 90)
    A = inputs.general_dominant_matrix(700, 42)
    got, _ = _gpu_lu(B, A, _fparams(B, 0, 1), want_info=False)
    _check_lu(oracle, got, A, 700)
    S = inputs.spd_matrix(700, 42)
    got, _ = _gpu_chol(B, S, _fparams(B, 0, 1), want_info=False)
    _check_chol(oracle, got, S, 700)


def test_a_partly_named_update_schedule_runs_as_tiled_gemms(B, oracle):
    """Any non-zero field of the update schedule selects the tiled GEMM (fields left 0 take the menu's defaults):
    a search that varies tile_k or unroll_k alone must not time the default kernel at every point."""
    announce("update schedule with tile_k only")
    n = 900
    A = inputs.general_dominant_matrix(n, 47)
    for tile in ((0, 0, 32), (0, 0, 0, 2)):
        for la in (0, 1):
            B.profile_enable(True)
            got, info = _gpu_lu(B, A, _fparams(B, 128, la, tile))
            B.profile_enable(False)
            _, bulk_launches, _ = B.profile_read(B.PHASE_UPDATE)
            _, gemm_launches, _ = B.profile_read(B.PHASE_GEMM)
            B.profile_read(B.PHASE_DIAG), B.profile_read(B.PHASE_TRSM)
            assert info == 0 and bulk_launches == 0 and gemm_launches > 0
            _check_lu(oracle, got, A, n)


# ------------------------------------------------------------------ layout, streams, determinism
def test_cholesky_ignores_upper_triangle(B, oracle):
    announce("cholesky upper junk")
    n = 301
    S = inputs.spd_matrix(n, 43)
    junk = np.tril(S) + np.triu(np.full((n, n), np.nan), 1)
    got, info = _gpu_chol(B, junk, _fparams(B, 64))
    assert info == 0
    _check_chol(oracle, got, S, n)


def test_leading_dimension_and_stream(B, oracle):
    import torch
    announce("lda > n, side stream")
    n, pad = 273, 11
    A = inputs.general_dominant_matrix(n, 44)
    buf = torch.full((n, n + pad), -3.0, dtype=torch.float64, device="cuda")
    buf[:, :n] = to_device(A)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        B.lu_factor(buf[:, :n], _fparams(B, 64))
    s.synchronize()
    out = to_host(buf)
    _check_lu(oracle, out[:, :n], A, n)
    assert np.all(out[:, n:] == -3.0)


def test_repeated_calls_are_bitwise_identical(B):
    announce("determinism")
    A = inputs.diag_dominant_matrix(1500, 45)
    a, _ = _gpu_lu(B, A)
    b, _ = _gpu_lu(B, A)
    assert np.array_equal(a, b)
    S = inputs.spd_matrix(1500, 45)
    a, _ = _gpu_chol(B, S)
    b, _ = _gpu_chol(B, S)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("kind,n", [("lu", 2100), ("chol", 2100), ("lu", 4000)])
def test_forty_calls_in_a_row_give_the_same_bits(B, kind, n):
    """The kernels of the latency chain hand their results over through memory while both still run; a
    hand-over that let a consumer read stale data would show as a run that differs.  Forty factorisations of
    one matrix, enqueued without synchronisation in between, compared on the device with the first."""
    import torch
    announce(f"forty calls {kind} n={n}")
    H = inputs.diag_dominant_matrix(n, 46) if kind == "lu" else inputs.spd_matrix(n, 46)
    src = to_device(H)
    fn = B.lu_factor if kind == "lu" else B.cholesky_factor
    ws = torch.empty(B.factor_workspace_bytes(n, B.DLA_F64, None), dtype=torch.uint8, device="cuda")
    info = torch.zeros(1, dtype=torch.int32, device="cuda")
    first = src.clone()
    fn(first, None, workspace=ws, info=info)
    work = torch.empty_like(src)
    differing = torch.zeros(1, dtype=torch.int64, device="cuda")
    for _ in range(40):
        work.copy_(src)
        fn(work, None, workspace=ws, info=info)
        differing += (work != first).sum()
    torch.cuda.synchronize()
    assert int(info.item()) == 0 and int(differing.item()) == 0


# ------------------------------------------------------------------ fp32 variant
@pytest.mark.parametrize("n,nb", [(500, 128), (1000, 64)])
def test_fp32_factorisations(B, oracle, n, nb):
    """fp32 kernels against the fp64 oracle applied to the fp32-rounded input."""
    import torch
    announce(f"fp32 n={n} nb={nb}")
    A32 = inputs.diag_dominant_matrix(n, 46).astype(np.float32)
    got, info = _gpu_lu(B, A32, _fparams(B, nb), dtype=torch.float32)
    assert info == 0 and got.dtype == np.float32
    _check_lu(oracle, got.astype(np.float64), A32.astype(np.float64), n, TOL32, EPS32)
    S32 = inputs.spd_matrix(n, 47).astype(np.float32)
    got, info = _gpu_chol(B, S32, _fparams(B, nb), dtype=torch.float32)
    assert info == 0
    _check_chol(oracle, got.astype(np.float64), S32.astype(np.float64), n, TOL32, EPS32)


def test_n8192_fp32_properties(B, oracle):
    """The fp32 variant at N=8192, block size 128: exact all-ones factors of the min-index matrix (every
    intermediate is an integer below 2^24); for the seeded inputs rounded to fp32, randomised reconstruction
    checks with the oracle's fp64 matrix-vector routines, and the factors element by element against the
    fp64 oracle's factorisation of the same fp32-rounded matrix."""
    import torch
    n = 8192
    announce("fp32 N=8192 min-index exact")
    A = inputs.min_index_matrix(n)
    got, info = _gpu_lu(B, A, dtype=torch.float32)
    assert info == 0 and got.dtype == np.float32 and np.array_equal(got, np.ones((n, n), dtype=np.float32))
    got, info = _gpu_chol(B, A, dtype=torch.float32)
    assert info == 0 and np.array_equal(got, np.tril(np.ones((n, n), dtype=np.float32)))
    del A, got
    announce("fp32 N=8192 LU reconstruction")
    A32 = inputs.diag_dominant_matrix(n, 6).astype(np.float32)
    lu, info = _gpu_lu(B, A32, dtype=torch.float32)
    assert info == 0
    A64, lu64 = A32.astype(np.float64), lu.astype(np.float64)
    for t in range(3):
        x = inputs.uniform_matrix(6, 70 + t, n, 1).ravel()
        y0, y1 = oracle.matvec(A64, x), oracle.lu_apply(lu64, x)
        assert np.linalg.norm(y0 - y1) <= 10 * n * EPS32 * np.linalg.norm(y0)
    announce("fp32 N=8192 LU element by element against the fp64 oracle on the fp32-rounded input")
    want, winfo = oracle.lu(A64)
    assert winfo == 0 and lu_rel_err(lu64, want) <= TOL32
    del lu, lu64, want
    announce("fp32 N=8192 Cholesky reconstruction")
    A64[np.diag_indices(n)] += 1.0 - float(n)  # the SPD generator: same Gram matrix, +I
    S32 = A64.astype(np.float32)
    L, info = _gpu_chol(B, S32, dtype=torch.float32)
    assert info == 0 and np.all(np.triu(L, 1) == 0.0)
    S64, L64 = S32.astype(np.float64), L.astype(np.float64)
    for t in range(3):
        x = inputs.uniform_matrix(6, 80 + t, n, 1).ravel()
        y0, y1 = oracle.symv_lower(S64, x), oracle.cholesky_apply(L64, x)
        assert np.linalg.norm(y0 - y1) <= 10 * n * EPS32 * np.linalg.norm(y0)
    announce("fp32 N=8192 Cholesky element by element against the fp64 oracle on the fp32-rounded input")
    want, winfo = oracle.cholesky(S64)
    assert winfo == 0 and cholesky_rel_err(L64, want) <= TOL32


@pytest.mark.parametrize("m,k", [(1, 1), (17, 16), (200, 48), (333, 128), (1000, 128), (2081, 96),
                                 (300, 256), (1000, 200), (777, 144),   # depth above 128: the two-panel form
                                 (1952, 256), (2080, 128),              # a last row panel with waves below the matrix
                                 (6200, 256), (6333, 128)])  # large: row-split launches (LU), panel-crossing items (Cholesky)
@pytest.mark.parametrize("lower", [False, True])
def test_rank_update_alone(B, oracle, m, k, lower):
    """dla_rank_update (the bulk trailing update on its own) against the oracle's plain product (the E of a
    3mm whose second product is empty-sized): ragged row panels, ragged column blocks, partial k."""
    import torch
    announce(f"rank_update m={m} k={k} lower={lower}")
    n = m + k
    A = inputs.uniform_matrix(11, 3, n, n)
    a = to_device(A)
    L, R, C = a[k:, :k], a[:k, k:], a[k:, k:]
    B.dla_rank_update(lower, L, R, C)
    torch.cuda.synchronize()
    got = to_host(a)
    exp = A.copy()
    def product(X, Y):
        return oracle_product(oracle, X, Y)

    if lower:
        full = A[k:, k:] - product(A[k:, :k], np.ascontiguousarray(A[k:, :k].T))
        for r0 in range(0, m, 128):  # row block i is updated in columns 0 .. 128*(i+1)-1
            r1, c1 = min(r0 + 128, m), min(r0 + 128, m)
            exp[k + r0:k + r1, k:k + c1] = full[r0:r1, :c1]
    else:
        exp[k:, k:] = A[k:, k:] - product(A[k:, :k], A[:k, k:])
    assert np.array_equal(got[:k, :], A[:k, :]) and np.array_equal(got[:, :k], A[:, :k]), "operands must stay untouched"
    assert max_rel_err(got[k:, k:], exp[k:, k:]) <= TOL64


@pytest.mark.parametrize("m,k", [(1952, 256), (2080, 128), (333, 128), (300, 256)])
@pytest.mark.parametrize("lower", [False, True])
def test_rank_update_leaves_the_rows_below_the_matrix_alone(B, oracle, m, k, lower):
    """The last row panel of an update is partial: its waves below the matrix (and the lanes of a wave that straddles
    the last row) must neither store nor count on what lies there.  The matrix is followed in memory by guard rows
    of NaN; they must still be NaN bit for bit afterwards, and the result must not have picked any up."""
    import torch
    announce(f"rank_update with guard rows m={m} k={k} lower={lower}")
    n = m + k
    guard = 160  # more than the 128 rows of a row panel
    A = inputs.uniform_matrix(11, 5, n, n)
    a = torch.full((n + guard, n), float("nan"), dtype=torch.float64, device="cuda")
    a[:n].copy_(torch.from_numpy(A))
    L, R, C = a[k:n, :k], a[:k, k:], a[k:n, k:]
    B.dla_rank_update(lower, L, R, C)
    torch.cuda.synchronize()
    got = a.cpu().numpy()
    assert np.isnan(got[n:]).all(), "rows below the matrix were written"
    assert not np.isnan(got[:n]).any(), "the update read rows below the matrix into its result"
    if not lower:
        exp = A[k:, k:] - oracle_product(oracle, A[k:, :k], A[:k, k:])
        assert max_rel_err(got[k:n, k:], exp) <= TOL64


def test_back_to_back_calls_share_the_helper_streams(B, oracle):
    """Five factorisations of different sizes and kinds enqueued on one side stream without any
    synchronisation in between (the look-ahead helper streams and events are shared by all calls):
    every result must still match the oracle."""
    import torch
    announce("back-to-back mixed calls, no sync in between")
    cases = [("lu", 700, 128), ("chol", 517, 64), ("lu", 300, 48), ("chol", 1000, 128), ("lu", 129, 16)]
    hosts, devs = [], []
    for kind, n, nb in cases:
        H = inputs.general_dominant_matrix(n, 60 + n) if kind == "lu" else inputs.spd_matrix(n, 60 + n)
        hosts.append(H)
        devs.append(to_device(H))
    ws = torch.empty(B.factor_workspace_bytes(1000, B.DLA_F64, None), dtype=torch.uint8, device="cuda")
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        for (kind, n, nb), d in zip(cases, devs):
            fn = B.lu_factor if kind == "lu" else B.cholesky_factor
            fn(d, _fparams(B, nb), workspace=ws)
    s.synchronize()
    for (kind, n, nb), H, d in zip(cases, hosts, devs):
        if kind == "lu":
            _check_lu(oracle, to_host(d), H, n)
        else:
            _check_chol(oracle, to_host(d), H, n)


def test_two_host_threads_factor_at_the_same_time(B, oracle):
    """Two host threads, each with its own stream, matrices and workspace, call the factorisations at the same
    time (the binding releases the interpreter lock inside the calls).  The library lines the calls up on its
    shared helper streams; every result matches the oracle and no wait gives up."""
    import threading
    import torch
    announce("two host threads factor concurrently")
    jobs = [("lu", 1500, 70), ("chol", 1300, 71), ("lu", 900, 72), ("chol", 1000, 73)]
    hosts = [inputs.general_dominant_matrix(n, s) if k == "lu" else inputs.spd_matrix(n, s) for k, n, s in jobs]
    devs = [to_device(H) for H in hosts]
    infos = [torch.full((1,), -99, dtype=torch.int32, device="cuda") for _ in jobs]
    wss = [torch.empty(B.factor_workspace_bytes(n, B.DLA_F64, None), dtype=torch.uint8, device="cuda") for _, n, _ in jobs]
    torch.cuda.synchronize()
    errors = []

    def worker(idx):
        try:
            st = torch.cuda.Stream()
            for rep in range(3):
                for j in idx:
                    if rep:
                        with torch.cuda.stream(st):
                            devs[j].copy_(torch.from_numpy(hosts[j]).to("cuda"))
                    fn = B.lu_factor if jobs[j][0] == "lu" else B.cholesky_factor
                    fn(devs[j], None, workspace=wss[j], info=infos[j], stream=st)
            st.synchronize()
        except Exception as e:  # surfaced in the main thread
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(idx,)) for idx in ((0, 1), (2, 3))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for (kind, n, _), H, d, info in zip(jobs, hosts, devs, infos):
        assert int(info.item()) == 0
        if kind == "lu":
            _check_lu(oracle, to_host(d), H, n)
        else:
            _check_chol(oracle, to_host(d), H, n)


def test_a_wait_that_cannot_end_gives_up_and_is_reported(B, oracle):
    """The pipeline's in-kernel wait is bounded: with nothing to wait for, the kernel ends after the poll and
    reports -1 (forced from the host: the counter it polls is never touched; every wave exits normally).
    A normal factorisation right after it is unaffected."""
    import time
    announce("hand-over self-test")
    t0 = time.perf_counter()
    assert B.handover_selftest() == -1
    assert time.perf_counter() - t0 < 5.0
    A = inputs.diag_dominant_matrix(700, 41)
    got, info = _gpu_lu(B, A)
    assert info == 0
    _check_lu(oracle, got, A, 700)
