// Host driver of the solves with the factors: A X = B as  L Y = B, U X = Y  (LU) or
// L Y = B, L^T X = Y  (Cholesky), B overwritten by X.  Blocked substitution over row blocks of up
// to 128: a pre-pass prepares every diagonal block for both passes (tri_prepare_kernel), then per
// block the block's own triangular system on trisolve_kernel and one tiled GEMM that carries the
// solved rows into the rows still open (below in the forward pass, above in the backward pass).
#include "trisolve_kernel.hpp"
#include "host_common.hpp"

namespace dla {

template <typename T, int MODE>
static int launch_prepare(const TriPrepareArgs<T>& a, hipStream_t st) {
  auto kern = tri_prepare_kernel<T, MODE>;
  static bool attr_done = false;
  if (!attr_done) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            trisolve_lds_bytes<T>()) != hipSuccess)
      return DLA_ERR_HIP;
    attr_done = true;
  }
  const int grid = (int)((a.n + kNbMax - 1) / kNbMax);
  ProfileScope scope(PHASE_TRSM, 0.0, st);
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kTriThreads), trisolve_lds_bytes<T>(), st, a);
  return hipGetLastError() == hipSuccess ? DLA_SUCCESS : DLA_ERR_HIP;
}

template <typename T, bool REV>
static int launch_trisolve(const TriSolveArgs<T>& a, hipStream_t st) {
  auto kern = trisolve_kernel<T, REV>;
  static bool attr_done = false;
  if (!attr_done) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            trisolve_lds_bytes<T>()) != hipSuccess)
      return DLA_ERR_HIP;
    attr_done = true;
  }
  const int per_wg = (kTriThreads / 64) * kIb;  // right-hand sides one workgroup solves
  const int grid = (a.nrhs + per_wg - 1) / per_wg;
  ProfileScope scope(PHASE_TRSM, 0.0, st);
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kTriThreads), trisolve_lds_bytes<T>(), st, a);
  return hipGetLastError() == hipSuccess ? DLA_SUCCESS : DLA_ERR_HIP;
}

// Workspace: per diagonal block of the factor, the prepared block of the forward pass and the one
// of the backward pass.
size_t solve_workspace_bytes_impl(int64_t n, dla_dtype dt) {
  const size_t blocks = (size_t)((n + kNbMax - 1) / kNbMax);
  const size_t one = dt == DLA_F64 ? (size_t)trisolve_lds_bytes<double>() : (size_t)trisolve_lds_bytes<float>();
  return 2 * blocks * one;
}

template <typename T, int KIND>
int solve_impl(const T* F, int64_t n, int64_t lda, T* B, int64_t nrhs, int64_t ldb, void* ws, size_t ws_bytes,
               hipStream_t st) {
  if (n == 0 || nrhs == 0) return DLA_SUCCESS;
  const dla_dtype dt = sizeof(T) == 8 ? DLA_F64 : DLA_F32;
  if (!ws || ws_bytes < solve_workspace_bytes_impl(n, dt) || ((uintptr_t)ws % 256)) return DLA_ERR_WORKSPACE;
  constexpr int FWD = (KIND == KIND_LU) ? TRI_LOWER_UNIT : TRI_LOWER;
  constexpr int BWD = (KIND == KIND_LU) ? TRI_UPPER : TRI_LOWER_TRANS;
  const int64_t nb = kNbMax;
  const int64_t blocks = (n + nb - 1) / nb;
  const int64_t one = trisolve_lds_bytes<T>() / (int64_t)sizeof(T);  // elements of one prepared block
  T* const fwd = static_cast<T*>(ws);
  T* const bwd = fwd + blocks * one;
  // the updates are skinny (k = 128, few columns): small tiles spread them over the compute units
  const GemmSchedule sch = nrhs <= 256 ? GemmSchedule{32, 32, 16, 4, 16, 16} : GemmSchedule{64, 64, 16, 2, 32, 32};
  int rc;
  if ((rc = launch_prepare<T, FWD>(TriPrepareArgs<T>{F, lda, n, fwd}, st)) != DLA_SUCCESS) return rc;
  if ((rc = launch_prepare<T, BWD>(TriPrepareArgs<T>{F, lda, n, bwd}, st)) != DLA_SUCCESS) return rc;
  auto block = [&](const T* prepared, int64_t k0) {
    TriSolveArgs<T> a;
    a.M = prepared + (k0 / nb) * one;
    a.B = B + k0 * ldb;
    a.ldb = ldb;
    a.b = (int)((n - k0 < nb) ? n - k0 : nb);
    a.nrhs = (int)nrhs;
    return a;
  };
  // forward: Y_k = L_kk^-1 B_k, then B_i -= L_ik Y_k for the rows i below
  for (int64_t k0 = 0; k0 < n; k0 += nb) {
    const TriSolveArgs<T> a = block(fwd, k0);
    if ((rc = launch_trisolve<T, false>(a, st)) != DLA_SUCCESS) return rc;
    const int64_t below = n - k0 - a.b;
    if (below > 0 && (rc = run_gemm<T>(sch, OP_SUB, F + (k0 + a.b) * lda + k0, lda, a.B, ldb, B + (k0 + a.b) * ldb, ldb,
                                       below, nrhs, a.b, st)) != DLA_SUCCESS)
      return rc;
  }
  // backward: X_k = U_kk^-1 Y_k, then B_i -= U_ik X_k for the rows i above (Cholesky: U = L^T,
  // read from L's block row k as a transposed left operand)
  for (int64_t k0 = (n - 1) / nb * nb; k0 >= 0; k0 -= nb) {
    const TriSolveArgs<T> a = block(bwd, k0);
    if ((rc = launch_trisolve<T, true>(a, st)) != DLA_SUCCESS) return rc;
    if (k0 == 0) break;
    if (KIND == KIND_LU) rc = run_gemm<T>(sch, OP_SUB, F + k0, lda, a.B, ldb, B, ldb, k0, nrhs, a.b, st);
    else rc = run_gemm<T>(sch, OP_SUB_TN, F + k0 * lda, lda, a.B, ldb, B, ldb, k0, nrhs, a.b, st);
    if (rc != DLA_SUCCESS) return rc;
  }
  return DLA_SUCCESS;
}

template int solve_impl<double, KIND_LU>(const double*, int64_t, int64_t, double*, int64_t, int64_t, void*, size_t, hipStream_t);
template int solve_impl<float, KIND_LU>(const float*, int64_t, int64_t, float*, int64_t, int64_t, void*, size_t, hipStream_t);
template int solve_impl<double, KIND_CHOL>(const double*, int64_t, int64_t, double*, int64_t, int64_t, void*, size_t, hipStream_t);
template int solve_impl<float, KIND_CHOL>(const float*, int64_t, int64_t, float*, int64_t, int64_t, void*, size_t, hipStream_t);

}  // namespace dla
