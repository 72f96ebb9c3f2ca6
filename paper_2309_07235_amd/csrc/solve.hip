// Host driver of the solves with the factors: A X = B as  L Y = B, U X = Y  (LU) or
// L Y = B, L^T X = Y  (Cholesky), B overwritten by X.  Blocked substitution over row blocks of up
// to 256.  A pre-pass, independent of B, inverts every diagonal block for both passes: the 128-row
// blocks by tri_prepare_kernel, then pairs of them joined into the inverse of a 256-row block,
//   inv [ L1  0  ] = [  W1        0  ]        inv [ U1 U12 ] = [ V1  -V1 U12 V2 ]
//       [ L21 L2 ]   [ -W2 L21 W1  W2 ]            [ 0  U2  ]   [ 0    V2       ]
// by two small products per pair on the tiled GEMM, all pairs in grouped launches.  After that each
// block step of the chain is two products: the block's solution X_k = W_k * B_k, then the solved
// rows carried into the rows still open (below in the forward pass, above in the backward pass).
// The first product cannot run in place, so the passes ping-pong: the forward pass reads B and
// leaves Y in the workspace, the backward pass reads Y there and leaves X in B.
#include "trisolve_kernel.hpp"
#include "host_common.hpp"

namespace dla {

template <typename T, int MODE>
static int launch_prepare(const TriPrepareArgs<T>& a, hipStream_t st) {
  auto kern = tri_prepare_kernel<T, MODE>;
  static LdsLimitOnce lds_limit;
  if (!lds_limit.ensure(reinterpret_cast<const void*>(kern), trisolve_lds_bytes<T>())) return DLA_ERR_HIP;
  const int grid = (int)((a.n + kNbMax - 1) / kNbMax);
  ProfileScope scope(PHASE_TRSM, 0.0, st);
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kTriThreads), trisolve_lds_bytes<T>(), st, a);
  return launch_status(__func__);
}

template <typename T>
__global__ void solve_zero_kernel(T* p, int64_t count) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) p[i] = T(0);
}

// Workspace: per pair of diagonal blocks a 256 x 256 inverse for the forward and one for the
// backward pass and a 128 x 128 intermediate for each, then the n x nrhs intermediate Y (leading
// dimension nrhs rounded up to even).
static int64_t pairs_of(int64_t n) { return (n + kTriPair - 1) / kTriPair; }
static int64_t inverse_elems(int64_t n) { return 2 * pairs_of(n) * ((int64_t)kTriPair * kTriPair + (int64_t)kNbMax * kNbMax); }
static int64_t y_ld(int64_t nrhs) { return (nrhs + 1) / 2 * 2; }
size_t solve_workspace_bytes_impl(int64_t n, int64_t nrhs, dla_dtype dt) {
  return ((size_t)inverse_elems(n) + (size_t)n * (size_t)y_ld(nrhs)) * (dt == DLA_F64 ? 8 : 4);
}

// products of one op and schedule, kMaxGroup to a launch
template <typename T>
struct ProductList {
  GemmSchedule sch;
  int op;
  GemmGroup<T> g;
  int np = 0, tiles = 0;
  double flops = 0.0;
  int flush(hipStream_t st) {
    if (np == 0) return DLA_SUCCESS;
    for (int q = np; q < kMaxGroup; ++q) g.prob[q] = g.prob[0];
    g.nprob = np;
    g.total_tiles = tiles;
    int rc;
    {
      ProfileScope scope(PHASE_GEMM, flops, st);
      rc = launch_gemm<T>(sch, op, g, st);
    }
    np = tiles = 0;
    flops = 0.0;
    return rc;
  }
  int add(const T* a, int64_t lda, const T* b, int64_t ldb, T* c, int64_t ldc, int64_t M, int64_t N, int64_t K,
          hipStream_t st) {
    if (M <= 0 || N <= 0 || K <= 0) return DLA_SUCCESS;
    g.prob[np] = make_problem<T>(sch, op, a, lda, b, ldb, c, ldc, M, N, K, tiles);
    tiles += problem_tiles(sch, op, g.prob[np]);
    flops += 2.0 * (double)M * (double)N * (double)K;
    if (++np == kMaxGroup) return flush(st);
    return DLA_SUCCESS;
  }
};

template <typename T, int KIND>
int solve_impl(const T* F, int64_t n, int64_t lda, T* B, int64_t nrhs, int64_t ldb, void* ws, size_t ws_bytes,
               hipStream_t st) {
  if (n == 0 || nrhs == 0) return DLA_SUCCESS;
  const dla_dtype dt = sizeof(T) == 8 ? DLA_F64 : DLA_F32;
  if (!ws || ws_bytes < solve_workspace_bytes_impl(n, nrhs, dt) || ((uintptr_t)ws % 256)) return DLA_ERR_WORKSPACE;
  constexpr int FWD = (KIND == KIND_LU) ? TRI_LOWER_UNIT : TRI_LOWER;
  constexpr int BWD = (KIND == KIND_LU) ? TRI_UPPER : TRI_LOWER_TRANS;
  const int64_t nb = kNbMax, sb = kTriPair;
  const int64_t pairs = pairs_of(n);
  T* const wf = static_cast<T*>(ws);      // inverses, forward pass: pairs x (256 x 256)
  T* const wb = wf + pairs * sb * sb;     // inverses, backward pass
  T* const tf = wb + pairs * sb * sb;     // intermediates of the pairing: pairs x (128 x 128), forward
  T* const tb = tf + pairs * nb * nb;     // and backward
  T* const Y = tb + pairs * nb * nb;      // n x nrhs
  const int64_t ldy = y_ld(nrhs);
  // the products are skinny (k <= 256, few columns): small tiles spread them over the compute units
  const GemmSchedule small = GemmSchedule{32, 32, 16, 4, 16, 16};
  const GemmSchedule sch = nrhs <= 256 ? small : GemmSchedule{64, 64, 16, 2, 32, 32};
  int rc;
  // ---- pre-pass: what the pairing leaves untouched must read as zero
  if (n > nb) {
    const int64_t count = inverse_elems(n);
    hipLaunchKernelGGL(solve_zero_kernel<T>, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, wf, count);
    if (launch_status(__func__) != DLA_SUCCESS) return DLA_ERR_HIP;
  }
  if ((rc = launch_prepare<T, FWD>(TriPrepareArgs<T>{F, lda, n, wf}, st)) != DLA_SUCCESS) return rc;
  if ((rc = launch_prepare<T, BWD>(TriPrepareArgs<T>{F, lda, n, wb}, st)) != DLA_SUCCESS) return rc;
  if (n > nb) {
    // T = -(off-diagonal block of the factor) * (inverse next to it), then the missing quarter = (the
    // other inverse) * T; the subtracting products start from the zeroed intermediates
    ProductList<T> first{small, OP_SUB}, first_t{small, OP_SUB_TN}, second{small, OP_ASSIGN};
    for (int pass = 0; pass < 2; ++pass) {
      for (int64_t p = 0; p < pairs; ++p) {
        const int64_t k0 = p * sb, b2 = n - k0 - nb < nb ? n - k0 - nb : nb;
        if (b2 <= 0) continue;  // a last block without a partner
        T* const W = (pass == 0 ? wf : wb) + p * sb * sb;
        T* const Tm = (pass == 0 ? tf : tb) + p * nb * nb;
        const T* const W1 = W;
        const T* const W2 = W + nb * sb + nb;
        const T* const L21 = F + (k0 + nb) * lda + k0;  // b2 x 128
        const T* const U12 = F + k0 * lda + k0 + nb;    // 128 x b2
        if (pass == 0) rc = first.add(L21, lda, W1, sb, Tm, nb, b2, nb, nb, st);            // T = -L21 W1
        else if (KIND == KIND_LU) rc = first.add(U12, lda, W2, sb, Tm, nb, nb, b2, b2, st);  // T = -U12 V2
        else rc = first_t.add(L21, lda, W2, sb, Tm, nb, nb, b2, b2, st);                     // T = -L21^T V2
        if (rc != DLA_SUCCESS) return rc;
      }
      if ((rc = first.flush(st)) != DLA_SUCCESS || (rc = first_t.flush(st)) != DLA_SUCCESS) return rc;
      for (int64_t p = 0; p < pairs; ++p) {
        const int64_t k0 = p * sb, b2 = n - k0 - nb < nb ? n - k0 - nb : nb;
        if (b2 <= 0) continue;
        T* const W = (pass == 0 ? wf : wb) + p * sb * sb;
        const T* const Tm = (pass == 0 ? tf : tb) + p * nb * nb;
        if (pass == 0) rc = second.add(W + nb * sb + nb, sb, Tm, nb, W + nb * sb, sb, b2, nb, b2, st);  // W21 = W2 T
        else rc = second.add(W, sb, Tm, nb, W + nb, sb, nb, b2, nb, st);                                 // W12 = V1 T
        if (rc != DLA_SUCCESS) return rc;
      }
      if ((rc = second.flush(st)) != DLA_SUCCESS) return rc;
    }
  }
  // ---- forward: Y_k = inv(L_kk) B_k, then B_i -= L_ik Y_k for the rows i below
  for (int64_t k0 = 0; k0 < n; k0 += sb) {
    const int64_t b = (n - k0 < sb) ? n - k0 : sb;
    T* const Yk = Y + k0 * ldy;
    if ((rc = run_gemm<T>(sch, OP_ASSIGN, wf + (k0 / sb) * sb * sb, sb, B + k0 * ldb, ldb, Yk, ldy, b, nrhs, b, st)) !=
        DLA_SUCCESS)
      return rc;
    const int64_t below = n - k0 - b;
    if (below > 0 && (rc = run_gemm<T>(sch, OP_SUB, F + (k0 + b) * lda + k0, lda, Yk, ldy, B + (k0 + b) * ldb, ldb, below,
                                       nrhs, b, st)) != DLA_SUCCESS)
      return rc;
  }
  // ---- backward: X_k = inv(U_kk) Y_k, then Y_i -= U_ik X_k for the rows i above (Cholesky: U = L^T,
  // read from L's block row k as a transposed left operand)
  for (int64_t k0 = (n - 1) / sb * sb; k0 >= 0; k0 -= sb) {
    const int64_t b = (n - k0 < sb) ? n - k0 : sb;
    T* const Xk = B + k0 * ldb;
    if ((rc = run_gemm<T>(sch, OP_ASSIGN, wb + (k0 / sb) * sb * sb, sb, Y + k0 * ldy, ldy, Xk, ldb, b, nrhs, b, st)) !=
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
