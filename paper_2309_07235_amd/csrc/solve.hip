// Host driver of the solves with the factors: A X = B as  L Y = B, U X = Y  (LU) or
// L Y = B, L^T X = Y  (Cholesky), B overwritten by X.  Blocked substitution over row blocks of up
// to 128.  A pre-pass inverts every diagonal block for both passes (tri_prepare_kernel); after that
// each block step is two products on the tiled GEMM: the block's solution X_k = W_k * B_k, then the
// solved rows carried into the rows still open (below in the forward pass, above in the backward
// pass).  The first product cannot run in place, so the passes ping-pong: the forward pass reads B
// and leaves Y in the workspace, the backward pass reads Y there and leaves X in B.
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

// Workspace: per diagonal block of the factor its 128 x 128 inverse for the forward and for the
// backward pass, then the n x nrhs intermediate Y (leading dimension nrhs rounded up to even).
static size_t inverse_bytes(int64_t n, dla_dtype dt) {
  const size_t blocks = (size_t)((n + kNbMax - 1) / kNbMax);
  return 2 * blocks * (size_t)kNbMax * kNbMax * (dt == DLA_F64 ? 8 : 4);
}
static int64_t y_ld(int64_t nrhs) { return (nrhs + 1) / 2 * 2; }
size_t solve_workspace_bytes_impl(int64_t n, int64_t nrhs, dla_dtype dt) {
  return inverse_bytes(n, dt) + (size_t)n * (size_t)y_ld(nrhs) * (dt == DLA_F64 ? 8 : 4);
}

template <typename T, int KIND>
int solve_impl(const T* F, int64_t n, int64_t lda, T* B, int64_t nrhs, int64_t ldb, void* ws, size_t ws_bytes,
               hipStream_t st) {
  if (n == 0 || nrhs == 0) return DLA_SUCCESS;
  const dla_dtype dt = sizeof(T) == 8 ? DLA_F64 : DLA_F32;
  if (!ws || ws_bytes < solve_workspace_bytes_impl(n, nrhs, dt) || ((uintptr_t)ws % 256)) return DLA_ERR_WORKSPACE;
  constexpr int FWD = (KIND == KIND_LU) ? TRI_LOWER_UNIT : TRI_LOWER;
  constexpr int BWD = (KIND == KIND_LU) ? TRI_UPPER : TRI_LOWER_TRANS;
  const int64_t nb = kNbMax;
  const int64_t blocks = (n + nb - 1) / nb;
  T* const wf = static_cast<T*>(ws);           // inverses, forward pass
  T* const wb = wf + blocks * nb * nb;         // inverses, backward pass
  T* const Y = wb + blocks * nb * nb;          // n x nrhs
  const int64_t ldy = y_ld(nrhs);
  // the products are skinny (k = 128, few columns): small tiles spread them over the compute units
  const GemmSchedule sch = nrhs <= 256 ? GemmSchedule{32, 32, 16, 4, 16, 16} : GemmSchedule{64, 64, 16, 2, 32, 32};
  int rc;
  if ((rc = launch_prepare<T, FWD>(TriPrepareArgs<T>{F, lda, n, wf}, st)) != DLA_SUCCESS) return rc;
  if ((rc = launch_prepare<T, BWD>(TriPrepareArgs<T>{F, lda, n, wb}, st)) != DLA_SUCCESS) return rc;
  // forward: Y_k = L_kk^-1 B_k, then B_i -= L_ik Y_k for the rows i below
  for (int64_t k0 = 0; k0 < n; k0 += nb) {
    const int64_t b = (n - k0 < nb) ? n - k0 : nb;
    T* const Yk = Y + k0 * ldy;
    if ((rc = run_gemm<T>(sch, OP_ASSIGN, wf + (k0 / nb) * nb * nb, nb, B + k0 * ldb, ldb, Yk, ldy, b, nrhs, b, st)) !=
        DLA_SUCCESS)
      return rc;
    const int64_t below = n - k0 - b;
    if (below > 0 && (rc = run_gemm<T>(sch, OP_SUB, F + (k0 + b) * lda + k0, lda, Yk, ldy, B + (k0 + b) * ldb, ldb, below,
                                       nrhs, b, st)) != DLA_SUCCESS)
      return rc;
  }
  // backward: X_k = U_kk^-1 Y_k, then Y_i -= U_ik X_k for the rows i above (Cholesky: U = L^T,
  // read from L's block row k as a transposed left operand)
  for (int64_t k0 = (n - 1) / nb * nb; k0 >= 0; k0 -= nb) {
    const int64_t b = (n - k0 < nb) ? n - k0 : nb;
    T* const Xk = B + k0 * ldb;
    if ((rc = run_gemm<T>(sch, OP_ASSIGN, wb + (k0 / nb) * nb * nb, nb, Y + k0 * ldy, ldy, Xk, ldb, b, nrhs, b, st)) !=
        DLA_SUCCESS)
      return rc;
    if (k0 == 0) break;
    if (KIND == KIND_LU) rc = run_gemm<T>(sch, OP_SUB, F + k0, lda, Xk, ldb, Y, ldy, k0, nrhs, b, st);
    else rc = run_gemm<T>(sch, OP_SUB_TN, F + k0 * lda, lda, Xk, ldb, Y, ldy, k0, nrhs, b, st);
    if (rc != DLA_SUCCESS) return rc;
  }
  return DLA_SUCCESS;
}

template int solve_impl<double, KIND_LU>(const double*, int64_t, int64_t, double*, int64_t, int64_t, void*, size_t, hipStream_t);
template int solve_impl<float, KIND_LU>(const float*, int64_t, int64_t, float*, int64_t, int64_t, void*, size_t, hipStream_t);
template int solve_impl<double, KIND_CHOL>(const double*, int64_t, int64_t, double*, int64_t, int64_t, void*, size_t, hipStream_t);
template int solve_impl<float, KIND_CHOL>(const float*, int64_t, int64_t, float*, int64_t, int64_t, void*, size_t, hipStream_t);

}  // namespace dla
