"""GPU parity of mm3 (and of the exported GEMM building block) against the CPU oracle."""
import numpy as np
import pytest

from paper_2309_07235_amd import inputs
from tests.gpu_util import announce, oracle_product, to_device, to_host
from tests.metrics import EPS32, EPS64, fro_rel_err, max_rel_err

pytestmark = pytest.mark.gpu

TOL64 = 1e-9   # max relative error bar for fp64 (denominator floored at the RMS of the expected entries)
TOL32 = 1e-4


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2309_07235_amd import binding
    return binding


def _run_mm3(B, ops, params=None, dtype=None):
    import torch
    A, Bm, C, D = (to_device(x, dtype) for x in ops)
    G = torch.full((A.shape[0], D.shape[1]), float("nan"), dtype=A.dtype, device="cuda")
    B.mm3(A, Bm, C, D, G, params)
    return to_host(G)


def _params(B, te, tf=None, tg=None):
    mk = lambda t: B.GemmParams(*t, *([0] * (6 - len(t))))
    return B.Mm3Params(mk(te), mk(tf or te), mk(tg or te))


def test_small_config_tiles_16x16(B, oracle):
    """3mm 128^3, all three products with 16x16 tiles."""
    announce("mm3 128^3 tiles 16x16")
    ops = inputs.mm3_operands(1, **inputs.MM3_SMALL)
    want = oracle.mm3(*ops)
    got = _run_mm3(B, ops, _params(B, (16, 16)))
    assert max_rel_err(got, want) <= TOL64
    assert fro_rel_err(got, want) <= 10 * 128 * EPS64


@pytest.mark.parametrize("dims", [(37, 53, 41, 29, 67), (1, 1, 1, 1, 1), (130, 17, 259, 5, 131), (16, 4, 16, 4, 16),
                                  (257, 129, 65, 33, 17)])
@pytest.mark.parametrize("tile", [(16, 16), (64, 64), (128, 128), (256, 128)])
def test_ragged_shapes(B, oracle, dims, tile):
    announce(f"mm3 ragged dims={dims} tile={tile}")
    ops = inputs.mm3_operands(11, *dims)
    want = oracle.mm3(*ops)
    got = _run_mm3(B, ops, _params(B, tile))
    assert max_rel_err(got, want) <= TOL64


def test_every_schedule_in_the_menu(B, oracle):
    """Each legal (tile, tile_k, unroll_k, wave split) on a shape with ragged edges in m, n and k."""
    dims = (150, 70, 210, 45, 139)
    ops = inputs.mm3_operands(12, *dims)
    want = oracle.mm3(*ops)
    dev = [to_device(x) for x in ops]
    import torch
    for t in B.enumerate_tiles(B.DLA_F64):
        announce(f"mm3 menu sweep {t}")
        G = torch.full((dims[0], dims[4]), float("nan"), dtype=torch.float64, device="cuda")
        B.mm3(*dev, G, B.Mm3Params(t, t, t))
        assert max_rel_err(to_host(G), want) <= TOL64, repr(t)


def test_mixed_schedules_per_product(B, oracle):
    """The three products may use three different schedules (the six parameters of the code mold)."""
    announce("mm3 mixed schedules")
    dims = (200, 90, 170, 110, 230)
    ops = inputs.mm3_operands(13, *dims)
    want = oracle.mm3(*ops)
    got = _run_mm3(B, ops, _params(B, (64, 64), (128, 64), (32, 32)))
    assert max_rel_err(got, want) <= TOL64


def test_integer_operands_are_bit_exact(B, oracle):
    """Entries in {-3..3}: every partial sum is an exact integer, so any summation order gives the same bits."""
    announce("mm3 integer exact 300x410x290x350x333")
    dims = (300, 410, 290, 350, 333)
    ops = inputs.mm3_integer_operands(14, *dims)
    want = oracle.mm3(*ops)
    for tile in ((128, 128), (64, 128), (16, 16)):
        got = _run_mm3(B, ops, _params(B, tile))
        assert np.array_equal(got, want), tile


def test_extralarge_config_full_size(B, oracle):
    """The rectangular extralarge shape, compared element by element at full size."""
    announce("mm3 extralarge 1600x2000x1800x2400x2200 default schedule")
    d = inputs.MM3_EXTRALARGE
    ops = inputs.mm3_operands(4, **d)
    want = oracle.mm3(*ops)
    got = _run_mm3(B, ops)
    assert max_rel_err(got, want) <= TOL64
    assert fro_rel_err(got, want) <= 10 * max(d["nk"], d["nj"], d["nm"]) * EPS64
    announce("mm3 extralarge integer operands, bit exact")
    iops = inputs.mm3_integer_operands(4, **d)
    assert np.array_equal(_run_mm3(B, iops), oracle.mm3(*iops))


def test_large_dataset(B, oracle):
    """The paper's "large" 3mm dataset: (N, L, M, O, P) = (800, 900, 1000, 1100, 1200)."""
    announce("mm3 large dataset")
    ops = inputs.mm3_operands(6, **inputs.MM3_LARGE_PAPER_ORDER)
    want = oracle.mm3(*ops)
    got = _run_mm3(B, ops)
    assert max_rel_err(got, want) <= TOL64
    assert fro_rel_err(got, want) <= 10 * 1100 * EPS64


def test_paper_literal_dimension_order(B, oracle):
    """The paper's own assignment of the five extralarge sizes (N, L, M, O, P) = (1600, 1800, 2000, 2200, 2400)."""
    announce("mm3 paper-order extralarge")
    ops = inputs.mm3_operands(5, **inputs.MM3_EXTRALARGE_PAPER_ORDER)
    want = oracle.mm3(*ops)
    assert max_rel_err(_run_mm3(B, ops), want) <= TOL64


def test_fp32_variant(B, oracle):
    """fp32 kernels against the fp64 oracle applied to the fp32-rounded inputs."""
    import torch
    announce("mm3 fp32 300x200x260x180x310")
    dims = (300, 200, 260, 180, 310)
    ops = [x.astype(np.float32) for x in inputs.mm3_operands(15, *dims)]
    want = oracle.mm3(*[x.astype(np.float64) for x in ops])
    for tile in ((128, 128), (32, 32), (256, 128)):
        got = _run_mm3(B, ops, _params(B, tile), dtype=torch.float32)
        assert got.dtype == np.float32
        assert max_rel_err(got, want) <= TOL32, tile


def test_degenerate_dimensions(B, oracle):
    import torch
    announce("mm3 degenerate dims")
    # nk == 0: E = 0 so G = 0;  nj == 0: G = 0;  ni == 0: empty G
    for dims in ((5, 0, 4, 3, 6), (5, 3, 0, 3, 6), (5, 3, 4, 0, 6)):
        ops = [np.ones(s) for s in ((dims[0], dims[1]), (dims[1], dims[2]), (dims[2], dims[3]), (dims[3], dims[4]))]
        got = _run_mm3(B, ops)
        assert got.shape == (5, 6) and np.all(got == 0.0), dims
    G = torch.empty((0, 6), dtype=torch.float64, device="cuda")
    B.mm3(to_device(np.ones((0, 3))), to_device(np.ones((3, 4))), to_device(np.ones((4, 3))),
          to_device(np.ones((3, 6))), G)
    torch.cuda.synchronize()


def test_strided_operands_and_stream(B, oracle):
    """Leading dimensions larger than the row length, odd leading dimension, and a non-default stream."""
    import torch
    announce("mm3 strided operands, side stream")
    dims = (70, 50, 60, 40, 90)
    ops = inputs.mm3_operands(16, *dims)
    want = oracle.mm3(*ops)
    dev = []
    for x, pad in zip(ops, (3, 1, 7, 5)):
        buf = torch.full((x.shape[0], x.shape[1] + pad), float("nan"), dtype=torch.float64, device="cuda")
        buf[:, :x.shape[1]] = to_device(x)
        dev.append(buf[:, :x.shape[1]])
    Gbuf = torch.full((dims[0], dims[4] + 9), -7.0, dtype=torch.float64, device="cuda")
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        B.mm3(*dev, Gbuf[:, :dims[4]])
    s.synchronize()
    got = to_host(Gbuf)
    assert max_rel_err(got[:, :dims[4]], want) <= TOL64
    assert np.all(got[:, dims[4]:] == -7.0)  # nothing written outside G


@pytest.mark.parametrize("op", [0, 1, 2, 3])
def test_gemm_building_block(B, oracle, op):
    """dla_gemm: assign, subtract, and the lower-triangular A*B^T update, against the oracle's plain product."""
    import torch
    announce(f"dla_gemm op={op}")
    m, n, k = (203, 203, 77) if op == 2 else (203, 157, 77)
    a = inputs.uniform_matrix(20, 0, m, k)
    b = inputs.uniform_matrix(20, 1, n, k) if op >= 2 else inputs.uniform_matrix(20, 1, k, n)
    c0 = inputs.uniform_matrix(20, 2, m, n)
    ab = oracle_product(oracle, a, b.T if op >= 2 else b)
    for tile in ((128, 128), (64, 64), (16, 16)):
        c = to_device(c0)
        B.dla_gemm(op, to_device(a), to_device(b), c, B.GemmParams(tile[0], tile[1], 0, 0, 0, 0))
        got = to_host(c)
        want = ab if op == 0 else c0 - ab  # op 2: lower tiles only, op 3: everywhere
        if op == 2:
            low = np.tril(np.ones((m, n), dtype=bool))
            assert max_rel_err(got[low], want[low]) <= TOL64
            # strictly-upper tiles are skipped: untouched there
            t = tile[0]
            for i in range(0, m, t):
                for j in range(i + t, n, t):
                    assert np.array_equal(got[i:i + t, j:j + t], c0[i:i + t, j:j + t])
        else:
            assert max_rel_err(got, want) <= TOL64
