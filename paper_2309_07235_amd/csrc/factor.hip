// Host drivers of the blocked right-looking factorisations: for every block
// column  (1) factor the diagonal block, (2) solve the panels, (3) update the
// trailing matrix with the MFMA GEMM (the step that dominates the run time).
#include "factor_kernels.hpp"
#include "host_common.hpp"

namespace dla {

static inline size_t round_up_sz(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Workspace: two parity sets of {inverted lower sub-blocks, inverted upper sub-blocks}.
static size_t inv_set_bytes(dla_dtype dt) {
  return round_up_sz((size_t)(kNbMax / kIb) * 256 * (dt == DLA_F64 ? 8 : 4), 256);
}

size_t factor_workspace_bytes_impl(int64_t n, dla_dtype dt, const dla_factor_params* p) {
  (void)n;
  (void)p;
  return 4 * inv_set_bytes(dt);
}

int resolve_factor_params(dla_dtype dt, int64_t n, const dla_factor_params* in, int op, int* nb, int* lookahead,
                          GemmSchedule* upd) {
  (void)n;
  int b = in ? in->nb : 0;
  if (b == 0) b = 128;
  if (b < 16 || b > kNbMax || b % 16 != 0) return DLA_ERR_UNSUPPORTED_PARAMS;
  int la = in ? in->lookahead : -1;
  if (la < -1 || la > 1) return DLA_ERR_UNSUPPORTED_PARAMS;
  if (la == -1) la = 0;
  *nb = b;
  *lookahead = la;
  return resolve_schedule(dt, in ? &in->update : nullptr, op, upd);
}

template <typename T, int KIND>
static int launch_diag(const DiagArgs<T>& a, hipStream_t st) {
  auto kern = diag_kernel<T, KIND>;
  static bool attr_done = false;
  if (!attr_done) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            diag_lds_bytes<T>()) != hipSuccess)
      return DLA_ERR_HIP;
    attr_done = true;
  }
  ProfileScope scope(PHASE_DIAG, 0.0, st);
  hipLaunchKernelGGL(kern, dim3(1), dim3(kDiagThreads), diag_lds_bytes<T>(), st, a);
  return hipGetLastError() == hipSuccess ? DLA_SUCCESS : DLA_ERR_HIP;
}

template <typename T, int KIND>
static int launch_trsm(TrsmArgs<T> a, hipStream_t st) {
  auto kern = trsm_kernel<T, KIND>;
  static bool attr_done = false;
  if (!attr_done) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            trsm_lds_bytes<T>()) != hipSuccess)
      return DLA_ERR_HIP;
    attr_done = true;
  }
  const int per_wg = (kTrsmThreads / 64) * kIb;  // panel rows/columns one workgroup solves
  const int wgs = (a.m + per_wg - 1) / per_wg;
  a.n_left = (KIND == KIND_LU) ? wgs : 0;
  const int grid = a.n_left + wgs;
  if (grid <= 0) return DLA_SUCCESS;
  ProfileScope scope(PHASE_TRSM, 0.0, st);
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kTrsmThreads), trsm_lds_bytes<T>(), st, a);
  return hipGetLastError() == hipSuccess ? DLA_SUCCESS : DLA_ERR_HIP;
}

template <typename T, int KIND>
static int factor_impl(T* A, int64_t n, int64_t lda, const dla_factor_params* p, void* ws, size_t ws_bytes,
                       hipStream_t st, int* d_info) {
  const dla_dtype dt = sizeof(T) == 8 ? DLA_F64 : DLA_F32;
  int nb, lookahead;
  GemmSchedule upd;
  const int op = (KIND == KIND_LU) ? OP_SUB : OP_SUB_NT_LOWER;
  int rc = resolve_factor_params(dt, n, p, op, &nb, &lookahead, &upd);
  if (rc != DLA_SUCCESS) return rc;
  if (n == 0) return DLA_SUCCESS;
  if (!ws || ws_bytes < factor_workspace_bytes_impl(n, dt, p) || ((uintptr_t)ws % 256)) return DLA_ERR_WORKSPACE;
  (void)lookahead;

  unsigned char* wsb = static_cast<unsigned char*>(ws);
  const size_t set = inv_set_bytes(dt);
  int step = 0;
  for (int64_t k0 = 0; k0 < n; k0 += nb, ++step) {
    const int b = (int)((n - k0 < nb) ? n - k0 : nb);
    const int64_t m = n - k0 - b;
    T* const Akk = A + k0 * lda + k0;
    T* const inv_lo = reinterpret_cast<T*>(wsb + (size_t)(2 * (step & 1)) * set);
    T* const inv_up = reinterpret_cast<T*>(wsb + (size_t)(2 * (step & 1) + 1) * set);

    DiagArgs<T> da;
    da.A = Akk;
    da.lda = lda;
    da.b = b;
    da.k0 = (int)k0;
    da.info = d_info;
    da.inv_lo = inv_lo;
    da.inv_up = inv_up;
    if ((rc = launch_diag<T, KIND>(da, st)) != DLA_SUCCESS) return rc;
    if (m == 0) break;

    TrsmArgs<T> ta;
    ta.D = Akk;
    ta.left = Akk + b;               // A12: b x m
    ta.right = Akk + (int64_t)b * lda;  // A21: m x b
    ta.lda = lda;
    ta.b = b;
    ta.m = (int)m;
    ta.n_left = 0;
    ta.inv_lo = inv_lo;
    ta.inv_up = inv_up;
    if ((rc = launch_trsm<T, KIND>(ta, st)) != DLA_SUCCESS) return rc;

    T* const A22 = Akk + (int64_t)b * lda + b;
    if (KIND == KIND_LU)
      rc = run_gemm<T>(upd, OP_SUB, ta.right, lda, ta.left, lda, A22, lda, m, m, b, st);
    else
      rc = run_gemm<T>(upd, OP_SUB_NT_LOWER, ta.right, lda, ta.right, lda, A22, lda, m, m, b, st);
    if (rc != DLA_SUCCESS) return rc;
  }
  if (KIND == KIND_CHOL && n > 1) {
    hipLaunchKernelGGL(zero_upper_kernel<T>, dim3((unsigned)((n + 255) / 256), (unsigned)(n < 32768 ? n : 32768)), dim3(256), 0, st, A, lda,
                       (int)n);
    if (hipGetLastError() != hipSuccess) return DLA_ERR_HIP;
  }
  return DLA_SUCCESS;
}

template <typename T>
int lu_factor_impl(T* A, int64_t n, int64_t lda, const dla_factor_params* p, void* ws, size_t ws_bytes,
                   hipStream_t st, int* d_info) {
  return factor_impl<T, KIND_LU>(A, n, lda, p, ws, ws_bytes, st, d_info);
}
template <typename T>
int cholesky_factor_impl(T* A, int64_t n, int64_t lda, const dla_factor_params* p, void* ws, size_t ws_bytes,
                         hipStream_t st, int* d_info) {
  return factor_impl<T, KIND_CHOL>(A, n, lda, p, ws, ws_bytes, st, d_info);
}

template int lu_factor_impl<double>(double*, int64_t, int64_t, const dla_factor_params*, void*, size_t, hipStream_t,
                                    int*);
template int lu_factor_impl<float>(float*, int64_t, int64_t, const dla_factor_params*, void*, size_t, hipStream_t,
                                   int*);
template int cholesky_factor_impl<double>(double*, int64_t, int64_t, const dla_factor_params*, void*, size_t,
                                          hipStream_t, int*);
template int cholesky_factor_impl<float>(float*, int64_t, int64_t, const dla_factor_params*, void*, size_t,
                                         hipStream_t, int*);

}  // namespace dla
