"""mm3_noalloc (E and F in the library's fixed device scratch, nothing allocated) against mm3 with a caller
workspace: same kernels, same schedules, so the results must agree bit for bit; and against the oracle."""
import numpy as np
import pytest

from paper_2309_07235_amd import inputs
from tests.gpu_util import announce, to_device, to_host
from tests.metrics import max_rel_err

pytestmark = pytest.mark.gpu

TOL64 = 1e-9


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2309_07235_amd import binding
    return binding


def _both(B, dims, seed, dtype=None):
    import torch
    ops = inputs.mm3_operands(seed, *dims)
    dev = [to_device(x, dtype) for x in ops]
    g_ws = torch.full((dims[0], dims[4]), -1.0, dtype=dev[0].dtype, device="cuda")
    g_na = torch.full((dims[0], dims[4]), -2.0, dtype=dev[0].dtype, device="cuda")
    B.mm3(*dev, g_ws)
    B.mm3_noalloc(*dev, g_na)
    return ops, to_host(g_ws), to_host(g_na)


def test_two_calls_in_a_row_the_second_smaller(B, oracle):
    """The scratch keeps the first call's E and F; the second, smaller call must not see them."""
    announce("mm3_noalloc 333x210x250x190x275, then 100x64x90x50x70")
    for seed, dims in ((51, (333, 210, 250, 190, 275)), (52, (100, 64, 90, 50, 70))):
        ops, with_ws, no_alloc = _both(B, dims, seed)
        assert np.array_equal(with_ws, no_alloc), dims
        assert max_rel_err(no_alloc, oracle.mm3(*ops)) <= TOL64


def test_fp32_and_ragged_shapes(B, oracle):
    import torch
    announce("mm3_noalloc fp32 150x70x210x45x139, then fp64 1x1x1x1x1")
    ops, with_ws, no_alloc = _both(B, (150, 70, 210, 45, 139), 53, torch.float32)
    assert no_alloc.dtype == np.float32 and np.array_equal(with_ws, no_alloc)
    ops64 = [x.astype(np.float32).astype(np.float64) for x in ops]
    assert max_rel_err(no_alloc.astype(np.float64), oracle.mm3(*ops64)) <= 1e-4
    ops, with_ws, no_alloc = _both(B, (1, 1, 1, 1, 1), 54)
    assert np.array_equal(with_ws, no_alloc) and max_rel_err(no_alloc, oracle.mm3(*ops)) <= TOL64


def test_extralarge_fits_and_too_large_is_refused(B):
    import torch
    announce("mm3_noalloc extralarge shape; 3000^3 refused")
    d = inputs.MM3_EXTRALARGE
    ops = inputs.mm3_integer_operands(55, **d)
    dev = [to_device(x) for x in ops]
    g_ws = torch.empty((d["ni"], d["nl"]), dtype=torch.float64, device="cuda")
    g_na = torch.empty_like(g_ws)
    B.mm3(*dev, g_ws)
    B.mm3_noalloc(*dev, g_na)
    torch.cuda.synchronize()
    assert torch.equal(g_ws, g_na)
    n = 3000
    z = torch.zeros((n, n), dtype=torch.float64, device="cuda")
    with pytest.raises(B.DlaError) as e:
        B.mm3_noalloc(z, z, z, z, torch.empty_like(z))
    assert e.value.code == B.DLA_ERR_TOO_LARGE
    # and a small call right after the refusal still works
    ops = inputs.mm3_operands(56, 40, 30, 20, 10, 50)
    dev = [to_device(x) for x in ops]
    g1 = torch.empty((40, 50), dtype=torch.float64, device="cuda")
    g2 = torch.empty_like(g1)
    B.mm3(*dev, g1)
    B.mm3_noalloc(*dev, g2)
    torch.cuda.synchronize()
    assert torch.equal(g1, g2)
