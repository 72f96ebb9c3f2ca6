"""ctypes binding of the C ABI declared in ``include/dla.h``.

Argument marshalling only: every function here has the name and the meaning of
the C entry point it calls, takes torch tensors (device memory) and the current
torch stream, and does no arithmetic of its own.  If the shared library has not
been built the import of this module fails with instructions; there is no CPU
fallback.
"""
from __future__ import annotations

import ctypes
from pathlib import Path

# torch first: its wheel carries a HIP runtime of its own, and the streams and device pointers handed to this
# library belong to that runtime.  Loaded after it, the library's reference to the runtime resolves to the copy
# already in the process; loaded before it, the process would hold two runtimes that do not know of each other.
import torch  # noqa: F401

_HERE = Path(__file__).resolve().parent
LIB_PATH = _HERE / "libdla_mi355x.so"

DLA_F64, DLA_F32 = 0, 1
DLA_SUCCESS, DLA_ERR_UNSUPPORTED_PARAMS, DLA_ERR_WORKSPACE, DLA_ERR_HIP, DLA_ERR_TOO_LARGE = 0, 1, 2, 3, 4
DLA_KERNEL_MM3, DLA_KERNEL_LU, DLA_KERNEL_CHOLESKY = 0, 1, 2
OP_ASSIGN, OP_SUB, OP_SUB_NT_LOWER = 0, 1, 2
PHASE_GEMM, PHASE_DIAG, PHASE_TRSM, PHASE_UPDATE = 0, 1, 2, 3


class GemmParams(ctypes.Structure):
    _fields_ = [("tile_m", ctypes.c_int), ("tile_n", ctypes.c_int), ("tile_k", ctypes.c_int),
                ("unroll_k", ctypes.c_int), ("wave_m", ctypes.c_int), ("wave_n", ctypes.c_int)]

    def as_tuple(self):
        return (self.tile_m, self.tile_n, self.tile_k, self.unroll_k, self.wave_m, self.wave_n)

    def __repr__(self):
        return "GemmParams(tile=%dx%d, tile_k=%d, unroll_k=%d, wave=%dx%d)" % (
            self.tile_m, self.tile_n, self.tile_k, self.unroll_k, self.wave_m, self.wave_n)


class FactorParams(ctypes.Structure):
    _fields_ = [("nb", ctypes.c_int), ("lookahead", ctypes.c_int), ("update", GemmParams),
                ("defer_min_rows", ctypes.c_int)]


class Mm3Params(ctypes.Structure):
    _fields_ = [("e", GemmParams), ("f", GemmParams), ("g", GemmParams)]


class DlaError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        detail = lib.dla_last_error_detail().decode() if code == DLA_ERR_HIP else ""
        super().__init__(f"{where}: code {code}: {strerror(code)}" + (f" [{detail}]" if detail else ""))


def _load() -> ctypes.CDLL:
    if not LIB_PATH.exists():
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2309_07235_amd.build` "
            "(hipcc, gfx950). There is no fallback path.")
    lib = ctypes.CDLL(str(LIB_PATH))
    vp, i64, ci, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
    lib.lu_factor.argtypes = [vp, i64, i64, ci, ctypes.POINTER(FactorParams), vp, sz, vp, vp]
    lib.lu_factor.restype = ci
    lib.cholesky_factor.argtypes = lib.lu_factor.argtypes
    lib.cholesky_factor.restype = ci
    lib.lu_solve.argtypes = [vp, i64, i64, vp, i64, i64, ci, vp, sz, vp]
    lib.solve_workspace_bytes.argtypes = [i64, i64, ci]
    lib.solve_workspace_bytes.restype = sz
    lib.lu_solve.restype = ci
    lib.cholesky_solve.argtypes = lib.lu_solve.argtypes
    lib.cholesky_solve.restype = ci
    for fn in (lib.lu_solve_prepared, lib.cholesky_solve_prepared):
        fn.argtypes = lib.lu_solve.argtypes
        fn.restype = ci
    for fn in (lib.lu_solve_prepare, lib.cholesky_solve_prepare):
        fn.argtypes = [vp, i64, i64, ci, vp, sz, vp]
        fn.restype = ci
    lib.factor_workspace_bytes.argtypes = [i64, ci, ctypes.POINTER(FactorParams)]
    lib.factor_workspace_bytes.restype = sz
    lib.mm3.argtypes = [vp, i64, vp, i64, vp, i64, vp, i64, vp, i64, i64, i64, i64, i64, i64, ci,
                        ctypes.POINTER(Mm3Params), vp, sz, vp]
    lib.mm3.restype = ci
    lib.mm3_noalloc.argtypes = [vp, i64, vp, i64, vp, i64, vp, i64, vp, i64, i64, i64, i64, i64, i64, ci,
                                ctypes.POINTER(Mm3Params), vp]
    lib.mm3_noalloc.restype = ci
    lib.mm3_workspace_bytes.argtypes = [i64, i64, i64, ci]
    lib.mm3_workspace_bytes.restype = sz
    lib.dla_gemm.argtypes = [ci, vp, i64, vp, i64, vp, i64, i64, i64, i64, ci, ctypes.POINTER(GemmParams), vp]
    lib.dla_gemm.restype = ci
    lib.dla_mfma_peak.argtypes = [ci, vp, ctypes.c_size_t, vp, ctypes.POINTER(ctypes.c_double)]
    lib.dla_mfma_peak.restype = ci
    lib.dla_mfma_peak_scratch_bytes.argtypes = []
    lib.dla_mfma_peak_scratch_bytes.restype = ctypes.c_size_t
    lib.dla_handover_selftest.argtypes = [vp, sz, vp, vp]
    lib.dla_handover_selftest.restype = ci
    lib.dla_rank_update.argtypes = [ci, vp, vp, vp, i64, i64, i64, ci, vp]
    lib.dla_rank_update.restype = ci
    lib.dla_gemm_params_supported.argtypes = [ci, ctypes.POINTER(GemmParams)]
    lib.dla_gemm_params_supported.restype = ci
    lib.dla_enumerate_tiles.argtypes = [ci, ctypes.POINTER(GemmParams), ci]
    lib.dla_enumerate_tiles.restype = ci
    lib.dla_block_size_supported.argtypes = [ci, ci]
    lib.dla_block_size_supported.restype = ci
    lib.dla_default_params.argtypes = [ci, i64, ci, vp]
    lib.dla_default_params.restype = ci
    lib.dla_profile_enable.argtypes = [ci]
    lib.dla_profile_enable.restype = ci
    lib.dla_profile_read.argtypes = [ci, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64),
                                     ctypes.POINTER(ctypes.c_double)]
    lib.dla_profile_read.restype = ci
    lib.dla_strerror.argtypes = [ci]
    lib.dla_strerror.restype = ctypes.c_char_p
    lib.dla_last_error_detail.argtypes = []
    lib.dla_last_error_detail.restype = ctypes.c_char_p
    lib.dla_version.argtypes = []
    lib.dla_version.restype = ctypes.c_char_p
    return lib


lib = _load()


def strerror(code: int) -> str:
    return lib.dla_strerror(int(code)).decode()


def version() -> str:
    return lib.dla_version().decode()


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float64:
        return DLA_F64
    if t.dtype == torch.float32:
        return DLA_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream_ptr(stream=None) -> int:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _matrix(t, name):
    if t.dim() != 2:
        raise ValueError(f"{name} must be a matrix")
    if t.numel() == 0:
        return ctypes.c_void_p(t.data_ptr() or None), int(max(t.shape[1], 1))
    if t.stride(1) != 1 and t.shape[1] > 1:
        raise ValueError(f"{name} must be a row-major matrix (unit column stride)")
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    ld = t.stride(0) if t.shape[0] > 1 else max(t.shape[1], 1)
    return ctypes.c_void_p(t.data_ptr()), int(max(ld, 1))


def _ref(p):
    return ctypes.byref(p) if p is not None else None


def _check(rc: int, where: str):
    if rc != DLA_SUCCESS:
        raise DlaError(rc, where)


def gemm_params_supported(dtype_code: int, p: GemmParams) -> bool:
    return bool(lib.dla_gemm_params_supported(dtype_code, ctypes.byref(p)))


def enumerate_tiles(dtype_code: int = DLA_F64):
    n = lib.dla_enumerate_tiles(dtype_code, None, 0)
    arr = (GemmParams * n)()
    lib.dla_enumerate_tiles(dtype_code, arr, n)
    return [GemmParams(*a.as_tuple()) for a in arr]


def block_size_supported(dtype_code: int, nb: int) -> bool:
    return bool(lib.dla_block_size_supported(dtype_code, nb))


def default_params(kernel: int, n: int, dtype_code: int = DLA_F64):
    out = Mm3Params() if kernel == DLA_KERNEL_MM3 else FactorParams()
    _check(lib.dla_default_params(kernel, n, dtype_code, ctypes.byref(out)), "dla_default_params")
    return out


def factor_workspace_bytes(n: int, dtype_code: int, p: FactorParams | None = None) -> int:
    return int(lib.factor_workspace_bytes(n, dtype_code, _ref(p)))


def mm3_workspace_bytes(ni: int, nj: int, nl: int, dtype_code: int) -> int:
    return int(lib.mm3_workspace_bytes(ni, nj, nl, dtype_code))


def _workspace(nbytes: int, device, workspace=None):
    import torch
    if workspace is None:
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
    return workspace, ctypes.c_void_p(workspace.data_ptr()), int(workspace.numel() * workspace.element_size())


def _factor(fn, name, a, p, workspace, info, stream):
    ap, lda = _matrix(a, "a")
    n = a.shape[0]
    if a.shape[1] != n:
        raise ValueError("a must be square")
    dt = _dtype_code(a)
    ws, wsp, wsb = _workspace(factor_workspace_bytes(n, dt, p), a.device, workspace)
    ip = ctypes.c_void_p(info.data_ptr()) if info is not None else None
    _check(fn(ap, n, lda, dt, _ref(p), wsp, wsb, ctypes.c_void_p(_stream_ptr(stream)), ip), name)
    return ws


def lu_factor(a, p: FactorParams | None = None, workspace=None, info=None, stream=None):
    """In-place LU without pivoting of the square device tensor ``a`` (see dla.h: lu_factor)."""
    return _factor(lib.lu_factor, "lu_factor", a, p, workspace, info, stream)


def cholesky_factor(a, p: FactorParams | None = None, workspace=None, info=None, stream=None):
    """In-place Cholesky factorisation of the square device tensor ``a`` (see dla.h: cholesky_factor)."""
    return _factor(lib.cholesky_factor, "cholesky_factor", a, p, workspace, info, stream)


def solve_workspace_bytes(n: int, nrhs: int, dt: int) -> int:
    return int(lib.solve_workspace_bytes(n, nrhs, dt))


def _solve(fn, name: str, f, b, workspace, stream):
    n = f.shape[0]
    if f.ndim != 2 or f.shape[1] != n:
        raise ValueError(f"{name}: the factor must be square")
    if b.ndim != 2 or b.shape[0] != n:
        raise ValueError(f"{name}: b must be a matrix with as many rows as the factor")
    dt = _dtype_code(f)
    if _dtype_code(b) != dt:
        raise ValueError(f"{name}: factor and right-hand sides differ in dtype")
    (fp, ldf), (bp, ldb) = _matrix(f, "factor"), _matrix(b, "b")
    ws, wsp, wsb = _workspace(solve_workspace_bytes(n, b.shape[1], dt), f.device, workspace)
    _check(fn(fp, n, ldf, bp, b.shape[1], ldb, dt, wsp, wsb, ctypes.c_void_p(_stream_ptr(stream))), name)
    return ws


def lu_solve(lu, b, workspace=None, stream=None):
    """Overwrites the device matrix b (n x nrhs) with X, (L*U)*X = b, from lu_factor's output (see dla.h: lu_solve).
    Returns the workspace it used (pass it back in to avoid the allocation)."""
    return _solve(lib.lu_solve, "lu_solve", lu, b, workspace, stream)


def cholesky_solve(l, b, workspace=None, stream=None):
    """Overwrites b with X, (L*L^T)*X = b, from cholesky_factor's output (see dla.h: cholesky_solve)."""
    return _solve(lib.cholesky_solve, "cholesky_solve", l, b, workspace, stream)


def _solve_prepare(fn, name: str, f, max_nrhs: int, workspace, stream):
    n = f.shape[0]
    if f.ndim != 2 or f.shape[1] != n:
        raise ValueError(f"{name}: the factor must be square")
    dt = _dtype_code(f)
    fp, ldf = _matrix(f, "factor")
    ws, wsp, wsb = _workspace(solve_workspace_bytes(n, max_nrhs, dt), f.device, workspace)
    _check(fn(fp, n, ldf, dt, wsp, wsb, ctypes.c_void_p(_stream_ptr(stream))), name)
    return ws


def lu_solve_prepare(lu, max_nrhs: int, workspace=None, stream=None):
    """The part of lu_solve that does not depend on the right-hand sides (see dla.h: lu_solve_prepare).  Returns the
    workspace, sized for up to max_nrhs right-hand sides, to pass to lu_solve_prepared."""
    return _solve_prepare(lib.lu_solve_prepare, "lu_solve_prepare", lu, max_nrhs, workspace, stream)


def cholesky_solve_prepare(l, max_nrhs: int, workspace=None, stream=None):
    """The part of cholesky_solve that does not depend on the right-hand sides (see dla.h: cholesky_solve_prepare)."""
    return _solve_prepare(lib.cholesky_solve_prepare, "cholesky_solve_prepare", l, max_nrhs, workspace, stream)


def lu_solve_prepared(lu, b, workspace, stream=None):
    """lu_solve with a workspace that lu_solve_prepare filled for this factor (see dla.h: lu_solve_prepared)."""
    if workspace is None:
        raise ValueError("lu_solve_prepared: pass the workspace lu_solve_prepare returned")
    return _solve(lib.lu_solve_prepared, "lu_solve_prepared", lu, b, workspace, stream)


def cholesky_solve_prepared(l, b, workspace, stream=None):
    """cholesky_solve with a workspace that cholesky_solve_prepare filled for this factor."""
    if workspace is None:
        raise ValueError("cholesky_solve_prepared: pass the workspace cholesky_solve_prepare returned")
    return _solve(lib.cholesky_solve_prepared, "cholesky_solve_prepared", l, b, workspace, stream)


def mm3(a, b, c, d, g, p: Mm3Params | None = None, workspace=None, stream=None):
    """G = (A*B)*(C*D) on device tensors; g is overwritten (see dla.h: mm3)."""
    ni, nk = a.shape
    nk2, nj = b.shape
    nj2, nm = c.shape
    nm2, nl = d.shape
    if nk != nk2 or nj != nj2 or nm != nm2 or tuple(g.shape) != (ni, nl):
        raise ValueError("3mm shapes do not chain")
    dt = _dtype_code(a)
    (ap, lda), (bp, ldb), (cp, ldc), (dp, ldd), (gp, ldg) = (_matrix(x, n) for x, n in
                                                             ((a, "a"), (b, "b"), (c, "c"), (d, "d"), (g, "g")))
    ws, wsp, wsb = _workspace(mm3_workspace_bytes(ni, nj, nl, dt), a.device, workspace)
    _check(lib.mm3(ap, lda, bp, ldb, cp, ldc, dp, ldd, gp, ldg, ni, nk, nj, nm, nl, dt, _ref(p), wsp, wsb,
                   ctypes.c_void_p(_stream_ptr(stream))), "mm3")
    return ws


MM3_NOALLOC_MAX_BYTES = 64 << 20


def mm3_noalloc(a, b, c, d, g, p: Mm3Params | None = None, stream=None):
    """mm3 with E and F in the library's fixed device scratch: no workspace, no allocation (see dla.h: mm3_noalloc)."""
    ni, nk = a.shape
    nk2, nj = b.shape
    nj2, nm = c.shape
    nm2, nl = d.shape
    if nk != nk2 or nj != nj2 or nm != nm2 or tuple(g.shape) != (ni, nl):
        raise ValueError("3mm shapes do not chain")
    dt = _dtype_code(a)
    (ap, lda), (bp, ldb), (cp, ldc), (dp, ldd), (gp, ldg) = (_matrix(x, n) for x, n in
                                                             ((a, "a"), (b, "b"), (c, "c"), (d, "d"), (g, "g")))
    _check(lib.mm3_noalloc(ap, lda, bp, ldb, cp, ldc, dp, ldd, gp, ldg, ni, nk, nj, nm, nl, dt, _ref(p),
                           ctypes.c_void_p(_stream_ptr(stream))), "mm3_noalloc")


def dla_gemm(op: int, a, b, c, p: GemmParams | None = None, stream=None):
    """c (op)= a*b with op 0: assign, 1: subtract, 2: lower(c) -= a*b^T, 3: c -= a*b^T, 4: c -= a^T*b
    (see dla.h: dla_gemm)."""
    m, k = (a.shape[1], a.shape[0]) if op == 4 else a.shape
    n = c.shape[1]
    dt = _dtype_code(a)
    (ap, lda), (bp, ldb), (cp, ldc) = _matrix(a, "a"), _matrix(b, "b"), _matrix(c, "c")
    _check(lib.dla_gemm(op, ap, lda, bp, ldb, cp, ldc, m, n, k, dt, _ref(p), ctypes.c_void_p(_stream_ptr(stream))),
           "dla_gemm")


def dla_rank_update(lower: bool, l, r, c, stream=None):
    """c -= l*r (lower False) or lower(c) -= l*l^T in 128-row blocks (lower True); see dla.h: dla_rank_update.
    l, r and c must share one leading dimension (views into one matrix)."""
    m, k = l.shape
    dt = _dtype_code(l)
    (lp, ldl), (cp, ldc) = _matrix(l, "l"), _matrix(c, "c")
    rp, ldr = (None, ldl) if lower else _matrix(r, "r")
    if not (ldl == ldc == ldr):
        raise ValueError("dla_rank_update: l, r and c must share one leading dimension")
    _check(lib.dla_rank_update(1 if lower else 0, lp, rp, cp, ldl, m, k, dt, ctypes.c_void_p(_stream_ptr(stream))),
           "dla_rank_update")


def handover_selftest(stream=None) -> int:
    """Runs the look-ahead pipeline's wait with nothing to wait for; returns what it reported (-1 expected)."""
    import torch
    scratch = torch.empty(8192, dtype=torch.uint8, device="cuda")
    info = torch.zeros(1, dtype=torch.int32, device="cuda")
    _check(lib.dla_handover_selftest(ctypes.c_void_p(scratch.data_ptr()), 8192, ctypes.c_void_p(_stream_ptr(stream)),
                                     ctypes.c_void_p(info.data_ptr())), "dla_handover_selftest")
    return int(info.item())


def mfma_peak(dt: int = DLA_F64, stream=None) -> float:
    """Achievable MFMA peak of the device in TFLOP/s for the given element type (see dla.h: dla_mfma_peak)."""
    import torch
    nbytes = int(lib.dla_mfma_peak_scratch_bytes())
    scratch = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    out = ctypes.c_double()
    _check(lib.dla_mfma_peak(dt, ctypes.c_void_p(scratch.data_ptr()), nbytes, ctypes.c_void_p(_stream_ptr(stream)),
                             ctypes.byref(out)), "dla_mfma_peak")
    return out.value


def profile_enable(on: bool) -> None:
    lib.dla_profile_enable(1 if on else 0)


def profile_read(phase: int):
    ms = ctypes.c_double()
    cnt = ctypes.c_int64()
    fl = ctypes.c_double()
    _check(lib.dla_profile_read(phase, ctypes.byref(ms), ctypes.byref(cnt), ctypes.byref(fl)), "dla_profile_read")
    return ms.value, cnt.value, fl.value
