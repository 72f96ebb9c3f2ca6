"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every function the public header declares, the schedule menu answers queries,
and argument errors are reported before any GPU work."""
import ctypes
import re
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
HEADER = ROOT / "include" / "dla.h"


@pytest.fixture(scope="module")
def B():
    from paper_2309_07235_amd import binding
    return binding


def _declared_functions():
    text = re.sub(r"/\*.*?\*/", "", HEADER.read_text(), flags=re.S)
    text = text.split('extern "C" {', 1)[1]
    names = re.findall(r"\b([a-z_0-9]+)\s*\([^;{}]*\)\s*;", text)
    return sorted(set(names))


def test_header_declares_the_boundary():
    names = _declared_functions()
    for must in ("lu_factor", "cholesky_factor", "lu_solve", "cholesky_solve", "mm3", "mm3_workspace_bytes",
                 "factor_workspace_bytes",
                 "dla_gemm", "dla_enumerate_tiles", "dla_gemm_params_supported", "dla_default_params",
                 "dla_strerror"):
        assert must in names


def test_library_exports_every_declared_symbol(B):
    for name in _declared_functions():
        assert hasattr(B.lib, name), f"{name} declared in dla.h but not exported"


def test_version_and_strerror(B):
    assert "gfx950" in B.version()
    assert B.strerror(0) == "success"
    assert "menu" in B.strerror(B.DLA_ERR_UNSUPPORTED_PARAMS)
    assert "argument" in B.strerror(-3)


def test_tile_menu_queries(B):
    tiles = B.enumerate_tiles(B.DLA_F64)
    assert len(tiles) >= 20
    shapes = {(t.tile_m, t.tile_n) for t in tiles}
    assert (16, 16) in shapes and (128, 128) in shapes  # the 16x16 tile of the small 3mm config is legal
    for t in tiles:
        assert B.gemm_params_supported(B.DLA_F64, t)
        assert t.tile_m % 16 == 0 and t.tile_n % 16 == 0 and t.tile_k % 4 == 0
    assert len(B.enumerate_tiles(B.DLA_F32)) >= len(tiles)  # fp32 tiles need less LDS
    # the paper's own candidates are divisors of the matrix size; most are not MFMA aligned and are refused
    for bad in ((5, 25), (125, 50), (400, 50), (1, 2000), (48, 48)):
        assert not B.gemm_params_supported(B.DLA_F64, B.GemmParams(bad[0], bad[1], 0, 0, 0, 0))
    assert B.gemm_params_supported(B.DLA_F64, B.GemmParams(0, 0, 0, 0, 0, 0))  # all defaults
    assert not B.gemm_params_supported(B.DLA_F64, B.GemmParams(128, 128, 12, 0, 0, 0))
    assert not B.gemm_params_supported(B.DLA_F64, B.GemmParams(256, 128, 32, 0, 0, 0))  # exceeds LDS in fp64
    assert B.gemm_params_supported(B.DLA_F32, B.GemmParams(256, 128, 32, 0, 0, 0))
    assert not B.gemm_params_supported(7, B.GemmParams(0, 0, 0, 0, 0, 0))


def test_block_sizes(B):
    legal = [nb for nb in range(0, 300) if B.block_size_supported(B.DLA_F64, nb)]
    assert legal == list(range(16, 129, 16)) + [160, 192, 224, 256]  # above 128: two sub-panels of nb / 2
    assert legal == [nb for nb in range(0, 300) if B.block_size_supported(B.DLA_F32, nb)]


def test_default_params(B):
    p = B.default_params(B.DLA_KERNEL_MM3, 2000)
    assert p.e.as_tuple() == p.f.as_tuple() == p.g.as_tuple()
    assert B.gemm_params_supported(B.DLA_F64, p.e)
    for k in (B.DLA_KERNEL_LU, B.DLA_KERNEL_CHOLESKY):
        f = B.default_params(k, 4000)
        assert B.block_size_supported(B.DLA_F64, f.nb)
        assert B.gemm_params_supported(B.DLA_F64, f.update)
        assert f.lookahead in (0, 1)


def test_workspace_queries(B):
    assert B.mm3_workspace_bytes(1600, 1800, 2200, B.DLA_F64) >= (1600 * 1800 + 1800 * 2200) * 8
    assert B.mm3_workspace_bytes(1600, 1800, 2200, B.DLA_F32) >= (1600 * 1800 + 1800 * 2200) * 4
    assert B.mm3_workspace_bytes(-1, 2, 3, B.DLA_F64) == 0
    assert B.factor_workspace_bytes(4000, B.DLA_F64) > 0
    assert B.factor_workspace_bytes(-1, B.DLA_F64) == 0


def test_argument_errors_are_reported_without_gpu_work(B):
    vp = ctypes.c_void_p
    fake = vp(0x1000)  # never dereferenced: every call below fails validation first
    L = B.lib
    assert L.lu_factor(None, 8, 8, B.DLA_F64, None, fake, 1 << 20, None, None) == -1
    assert L.lu_factor(fake, -1, 8, B.DLA_F64, None, fake, 1 << 20, None, None) == -2
    assert L.lu_factor(fake, 8, 7, B.DLA_F64, None, fake, 1 << 20, None, None) == -3
    assert L.lu_factor(fake, 8, 8, 5, None, fake, 1 << 20, None, None) == -4
    assert L.cholesky_factor(fake, 8, 4, B.DLA_F64, None, fake, 1 << 20, None, None) == -3
    assert L.lu_factor(vp(0x1004), 8, 8, B.DLA_F64, None, fake, 1 << 20, None, None) == -1  # misaligned
    bad = B.FactorParams(100, 0, B.GemmParams(0, 0, 0, 0, 0, 0))
    assert L.lu_factor(fake, 8, 8, B.DLA_F64, ctypes.byref(bad), fake, 1 << 20, None, None) == B.DLA_ERR_UNSUPPORTED_PARAMS
    for nb, la, tile, defer in ((144, 1, 0, 0), (272, 1, 0, 0), (256, 0, 0, 0), (192, 1, 64, 0), (128, 1, 0, -2)):
        # not a two-level size; too wide; two levels need the pipeline, and the default update kernel; bad threshold
        bad = B.FactorParams(nb, la, B.GemmParams(tile, tile, 0, 0, 0, 0), defer)
        assert L.lu_factor(fake, 8, 8, B.DLA_F64, ctypes.byref(bad), fake, 1 << 20, None, None) == B.DLA_ERR_UNSUPPORTED_PARAMS
    bad = B.FactorParams(64, 3, B.GemmParams(0, 0, 0, 0, 0, 0))  # look-ahead modes are 0, 1, 2
    assert L.lu_factor(fake, 8, 8, B.DLA_F64, ctypes.byref(bad), fake, 1 << 20, None, None) == B.DLA_ERR_UNSUPPORTED_PARAMS
    bad = B.FactorParams(64, 0, B.GemmParams(48, 48, 0, 0, 0, 0))
    assert L.cholesky_factor(fake, 8, 8, B.DLA_F64, ctypes.byref(bad), fake, 1 << 20, None, None) == B.DLA_ERR_UNSUPPORTED_PARAMS
    assert L.lu_factor(fake, 512, 512, B.DLA_F64, None, None, 0, None, None) == B.DLA_ERR_WORKSPACE
    assert L.lu_factor(fake, 512, 512, B.DLA_F64, None, fake, 16, None, None) == B.DLA_ERR_WORKSPACE
    # n == 0 is a successful no-op that touches nothing
    assert L.lu_factor(None, 0, 1, B.DLA_F64, None, None, 0, None, None) == 0
    assert L.cholesky_factor(None, 0, 1, B.DLA_F64, None, None, 0, None, None) == 0

    def mm3(a=fake, lda=8, b=fake, ldb=8, c=fake, ldc=8, d=fake, ldd=8, g=fake, ldg=8, dims=(8, 8, 8, 8, 8),
            dt=B.DLA_F64, p=None, ws=fake, wsb=1 << 20):
        return L.mm3(a, lda, b, ldb, c, ldc, d, ldd, g, ldg, *dims, dt, p, ws, wsb, None)

    assert mm3(a=None) == -1
    assert mm3(lda=7) == -2
    assert mm3(b=None) == -3
    assert mm3(ldb=3) == -4
    assert mm3(c=None) == -5
    assert mm3(ldc=3) == -6
    assert mm3(d=None) == -7
    assert mm3(ldd=3) == -8
    assert mm3(g=None) == -9
    assert mm3(ldg=3) == -10
    assert mm3(dims=(-1, 8, 8, 8, 8)) == -11
    assert mm3(dims=(8, 8, 8, 8, -2)) == -15
    assert mm3(dt=9) == -16
    assert mm3(ws=None) == B.DLA_ERR_WORKSPACE
    assert mm3(wsb=64) == B.DLA_ERR_WORKSPACE
    assert mm3(ws=vp(0x1008)) == B.DLA_ERR_WORKSPACE
    badp = B.Mm3Params(B.GemmParams(16, 16, 0, 0, 0, 0), B.GemmParams(5, 25, 0, 0, 0, 0), B.GemmParams(0, 0, 0, 0, 0, 0))
    assert mm3(p=ctypes.byref(badp)) == B.DLA_ERR_UNSUPPORTED_PARAMS
    assert mm3(dims=(0, 8, 8, 8, 8), a=None, g=None, ws=None, wsb=0) == 0  # empty G: nothing to do

    def mm3n(a=fake, lda=8, g=fake, ldg=8, dims=(8, 8, 8, 8, 8), dt=B.DLA_F64, p=None):
        return L.mm3_noalloc(a, lda, fake, 8, fake, 8, fake, 8, g, ldg, *dims, dt, p, None)

    # the entry point that allocates nothing: same argument checks, and sizes beyond its fixed scratch are refused
    assert mm3n(a=None) == -1
    assert mm3n(lda=7) == -2
    assert mm3n(g=None) == -9
    assert mm3n(dims=(8, 8, -1, 8, 8)) == -13
    assert mm3n(dt=9) == -16
    assert mm3n(p=ctypes.byref(badp)) == B.DLA_ERR_UNSUPPORTED_PARAMS
    big = (3000, 8, 3000, 8, 3000)  # E and F: 2 * 3000 * 3008 * 8 bytes > 64 MiB
    assert B.mm3_workspace_bytes(3000, 3000, 3000, B.DLA_F64) > B.MM3_NOALLOC_MAX_BYTES
    assert L.mm3_noalloc(fake, 8, fake, 3000, fake, 8, fake, 3000, fake, 3000, *big, B.DLA_F64, None, None) == B.DLA_ERR_TOO_LARGE
    assert B.mm3_workspace_bytes(1600, 1800, 2200, B.DLA_F64) <= B.MM3_NOALLOC_MAX_BYTES  # the extralarge 3mm fits
    assert mm3n(dims=(0, 8, 8, 8, 8), a=None, g=None) == 0  # empty G: nothing to do, the scratch is not looked up

    for solve in (L.lu_solve, L.cholesky_solve):
        assert solve(None, 8, 8, fake, 2, 2, B.DLA_F64, fake, 1 << 20, None) == -1
        assert solve(vp(0x1004), 8, 8, fake, 2, 2, B.DLA_F64, fake, 1 << 20, None) == -1  # misaligned
        assert solve(fake, -1, 8, fake, 2, 2, B.DLA_F64, fake, 1 << 20, None) == -2
        assert solve(fake, 8, 7, fake, 2, 2, B.DLA_F64, fake, 1 << 20, None) == -3
        assert solve(fake, 8, 8, None, 2, 2, B.DLA_F64, fake, 1 << 20, None) == -4
        assert solve(fake, 8, 8, fake, -2, 2, B.DLA_F64, fake, 1 << 20, None) == -5
        assert solve(fake, 8, 8, fake, 3, 2, B.DLA_F64, fake, 1 << 20, None) == -6
        assert solve(fake, 8, 8, fake, 2, 2, 7, fake, 1 << 20, None) == -7
        assert solve(fake, 8, 8, fake, 2, 2, B.DLA_F64, None, 0, None) == B.DLA_ERR_WORKSPACE
        assert solve(fake, 8, 8, fake, 2, 2, B.DLA_F64, fake, 64, None) == B.DLA_ERR_WORKSPACE
        assert solve(fake, 8, 8, fake, 2, 2, B.DLA_F64, vp(0x1008), 1 << 20, None) == B.DLA_ERR_WORKSPACE
        assert solve(None, 0, 1, None, 2, 2, B.DLA_F64, None, 0, None) == 0  # nothing to solve
        assert solve(fake, 8, 8, None, 0, 1, B.DLA_F64, None, 0, None) == 0  # no right-hand side
    for prep in (L.lu_solve_prepare, L.cholesky_solve_prepare):
        assert prep(None, 8, 8, B.DLA_F64, fake, 1 << 22, None) == -1
        assert prep(fake, -1, 8, B.DLA_F64, fake, 1 << 22, None) == -2
        assert prep(fake, 8, 7, B.DLA_F64, fake, 1 << 22, None) == -3
        assert prep(fake, 8, 8, 7, fake, 1 << 22, None) == -4
        assert prep(fake, 8, 8, B.DLA_F64, None, 0, None) == B.DLA_ERR_WORKSPACE
        assert prep(fake, 8, 8, B.DLA_F64, fake, L.solve_workspace_bytes(8, 0, B.DLA_F64) - 1, None) == B.DLA_ERR_WORKSPACE
        assert prep(None, 0, 1, B.DLA_F64, None, 0, None) == 0  # nothing to prepare
    for solve in (L.lu_solve_prepared, L.cholesky_solve_prepared):
        assert solve(None, 8, 8, fake, 2, 2, B.DLA_F64, fake, 1 << 22, None) == -1
        assert solve(fake, 8, 8, None, 2, 2, B.DLA_F64, fake, 1 << 22, None) == -4
        assert solve(fake, 8, 8, fake, 3, 2, B.DLA_F64, fake, 1 << 22, None) == -6
        assert solve(fake, 8, 8, fake, 2, 2, B.DLA_F64, fake, L.solve_workspace_bytes(8, 2, B.DLA_F64) - 1, None) == B.DLA_ERR_WORKSPACE
        assert solve(fake, 8, 8, None, 0, 1, B.DLA_F64, None, 0, None) == 0  # no right-hand side
    # per 256-row block and pass: a 256 x 256 inverse, a 128 x 128 intermediate, a 256 x 512 look-back product; two n x nrhs areas
    assert L.solve_workspace_bytes(4000, 63, B.DLA_F64) == (2 * 16 * (256 * 256 + 128 * 128 + 256 * 512) + 2 * 4000 * 64) * 8
    assert L.solve_workspace_bytes(1, 1, B.DLA_F32) == (2 * (256 * 256 + 128 * 128 + 256 * 512) + 2 * 2) * 4
    assert L.solve_workspace_bytes(-1, 1, B.DLA_F64) == 0 and L.solve_workspace_bytes(8, -1, B.DLA_F64) == 0
    assert L.solve_workspace_bytes(8, 1, 9) == 0
    assert L.dla_gemm(4, fake, 4, fake, 8, fake, 8, 8, 8, 8, B.DLA_F64, None, None) == -3  # A is k x m: lda >= m
    bad = B.GemmParams(128, 128, 16, 4, 64, 64)
    assert L.dla_gemm(4, fake, 8, fake, 8, fake, 8, 8, 8, 8, B.DLA_F64, ctypes.byref(bad), None) == B.DLA_ERR_UNSUPPORTED_PARAMS
    assert L.dla_gemm(7, fake, 8, fake, 8, fake, 8, 8, 8, 8, B.DLA_F64, None, None) == -1
    assert L.dla_gemm(0, None, 8, fake, 8, fake, 8, 8, 8, 8, B.DLA_F64, None, None) == -2
    assert L.dla_gemm(0, fake, 4, fake, 8, fake, 8, 8, 8, 8, B.DLA_F64, None, None) == -3
    assert L.dla_gemm(2, fake, 8, fake, 8, fake, 8, 8, 6, 8, B.DLA_F64, None, None) == -9
    assert L.dla_gemm(0, fake, 8, fake, 8, fake, 8, 0, 8, 8, B.DLA_F64, None, None) == 0
    assert L.dla_handover_selftest(None, 8192, None, fake) == -1
    assert L.dla_handover_selftest(fake, 100, None, fake) == -2
    assert L.dla_handover_selftest(fake, 8192, None, None) == -4
    assert L.dla_rank_update(2, fake, fake, fake, 256, 64, 16, B.DLA_F64, None) == -1
    assert L.dla_rank_update(0, None, fake, fake, 256, 64, 16, B.DLA_F64, None) == -2
    assert L.dla_rank_update(0, fake, None, fake, 256, 64, 16, B.DLA_F64, None) == -3
    assert L.dla_rank_update(1, fake, None, None, 256, 64, 16, B.DLA_F64, None) == -4
    assert L.dla_rank_update(0, fake, fake, fake, 32, 64, 16, B.DLA_F64, None) == -5
    assert L.dla_rank_update(0, fake, fake, fake, 256, -1, 16, B.DLA_F64, None) == -6
    assert L.dla_rank_update(0, fake, fake, fake, 512, 64, 257, B.DLA_F64, None) == -7
    assert L.dla_rank_update(0, fake, fake, fake, 256, 64, 16, 5, None) == -8
    assert L.dla_rank_update(0, fake, fake, fake, 256, 0, 16, B.DLA_F64, None) == 0
    tf = ctypes.c_double()
    assert L.dla_mfma_peak(7, fake, 1 << 22, None, ctypes.byref(tf)) == -1
    assert L.dla_mfma_peak(B.DLA_F64, None, 1 << 22, None, ctypes.byref(tf)) == -2
    assert L.dla_mfma_peak(B.DLA_F64, fake, 16, None, ctypes.byref(tf)) == B.DLA_ERR_WORKSPACE
    assert L.dla_mfma_peak(B.DLA_F64, fake, 1 << 22, None, None) == -5
    assert L.dla_mfma_peak_scratch_bytes() == 1024 * 256 * 8
    ms = ctypes.c_double()
    assert L.dla_profile_read(9, ctypes.byref(ms), None, None) == -1
