// Host driver of the solves with the factors: A X = B as  L Y = B, U X = Y  (LU) or
// L Y = B, L^T X = Y  (Cholesky), B overwritten by X.  Blocked substitution over row blocks of up
// to 256.  A pre-pass, independent of B, inverts every diagonal block: the 128-row blocks by
// tri_prepare_kernel, then pairs of them joined into the inverse of a 256-row block,
//   inv [ L1  0  ] = [  W1        0  ]        inv [ U1 U12 ] = [ V1  -V1 U12 V2 ]
//       [ L21 L2 ]   [ -W2 L21 W1  W2 ]            [ 0  U2  ]   [ 0    V2       ]
// by two small products per pair on the tiled GEMM, all pairs in grouped launches.
//
// The chain of the substitution is latency bound (every launch waits for the one before it), so a
// block step is ONE grouped launch.  With W_i the inverse of diagonal block i, the plain step
//   X_i = W_i (B_i - sum_{j<i} L_ij X_j)
// is split as  X_i = Z_i - M_i [X_{i-2}; X_{i-1}],  Z_i = W_i (B_i - sum_{j<i-2} L_ij X_j),
// M_i = W_i [L_{i,i-2}, L_{i,i-1}]  (the pre-pass forms M_i, one product per block).  The launch that
// follows X_k then carries three products that read nothing newer than X_k:
//   (a) X_{k+1} = Z_{k+1} - M_{k+1} [X_{k-1}; X_k]
//   (b) Z_{k+2} = W_{k+2} B_{k+2}            (B_{k+2} already holds the contributions of X_0..X_{k-1})
//   (c) B_i -= L_ik X_k  for the blocks i >= k + 3
// and the backward pass mirrors it from the last block upwards.  A launch has one operation for all
// its products, the subtracting one, so the pre-pass stores the NEGATED inverses N = -W and every
// product is  C -= A * B  on a target that starts at zero where a plain product is meant
// (Z = 0 - N B,  M = 0 - N L).  For Cholesky the backward inverse is the transpose of the forward one
// and the backward pass reads N, M^T and L's block rows as transposed left operands, so it needs no
// inverses of its own.  The forward pass leaves Y in the workspace and spoils B; the backward pass
// builds X in a second workspace area and stores each finished block to B as well.
// The chain's launches run on skinny_kernel up to 128 right-hand sides and on the tiled GEMM above.
// The pre-pass and the two passes can be called separately (one pre-pass, many solves with its workspace).
#include "trisolve_kernel.hpp"
#include "skinny_kernel.hpp"
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

template <typename T, int MODE_A, int MODE_B>
static int launch_prepare_both(const TriPrepareArgs<T>& a, const TriPrepareArgs<T>& b, hipStream_t st) {
  auto kern = tri_prepare_both_kernel<T, MODE_A, MODE_B>;
  static LdsLimitOnce lds_limit;
  if (!lds_limit.ensure(reinterpret_cast<const void*>(kern), trisolve_lds_bytes<T>())) return DLA_ERR_HIP;
  const int grid = 2 * (int)((a.n + kNbMax - 1) / kNbMax);
  ProfileScope scope(PHASE_TRSM, 0.0, st);
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kTriThreads), trisolve_lds_bytes<T>(), st, a, b);
  return launch_status(__func__);
}

template <typename T>
static int launch_skinny(bool at, const SkinnyGroup<T>& g, int workgroups, int kmax, double flops, hipStream_t st) {
  ProfileScope scope(PHASE_GEMM, flops, st);
  const dim3 grid((unsigned)workgroups), block(kSkinnyThreads);
  if (kmax <= 256) {
    if (at) hipLaunchKernelGGL((skinny_kernel<T, true, 16>), grid, block, 0, st, g);
    else hipLaunchKernelGGL((skinny_kernel<T, false, 16>), grid, block, 0, st, g);
  } else {
    if (at) hipLaunchKernelGGL((skinny_kernel<T, true, 32>), grid, block, 0, st, g);
    else hipLaunchKernelGGL((skinny_kernel<T, false, 32>), grid, block, 0, st, g);
  }
  return launch_status(__func__);
}

template <typename T>
__global__ void solve_zero_kernel(T* p, int64_t count) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) p[i] = T(0);
}

// Workspace, in elements: per 256-row block a 256 x 256 negated inverse for the forward and one for the
// backward pass (LU), a 128 x 128 intermediate of the pairing for each, and a 256 x 512 area M for each
// pass; then the n x nrhs areas Y and X (leading dimension nrhs rounded up to even).  All of it is
// cleared at the start of a call.
static int64_t pairs_of(int64_t n) { return (n + kTriPair - 1) / kTriPair; }
static int64_t block_elems(int64_t n) {
  return 2 * pairs_of(n) * ((int64_t)kTriPair * kTriPair + (int64_t)kNbMax * kNbMax + 2 * (int64_t)kTriPair * kTriPair);
}
static int64_t y_ld(int64_t nrhs) { return (nrhs + 1) / 2 * 2; }
size_t solve_workspace_bytes_impl(int64_t n, int64_t nrhs, dla_dtype dt) {
  return ((size_t)block_elems(n) + 2 * (size_t)n * (size_t)y_ld(nrhs)) * (dt == DLA_F64 ? 8 : 4);
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

// phases: kSolvePrepare = the pre-pass (independent of B; leaves the negated inverses and M in the workspace),
// kSolveApply = the two passes over B with a workspace the pre-pass has filled for this factor; both = a whole solve.
template <typename T, int KIND>
int solve_impl(const T* F, int64_t n, int64_t lda, T* B, int64_t nrhs, int64_t ldb, void* ws, size_t ws_bytes,
               hipStream_t st, int phases) {
  const bool prepare = phases & kSolvePrepare, apply = (phases & kSolveApply) && nrhs > 0;
  if (n == 0 || (nrhs == 0 && (phases & kSolveApply))) return DLA_SUCCESS;
  const dla_dtype dt = sizeof(T) == 8 ? DLA_F64 : DLA_F32;
  if (!ws || ws_bytes < solve_workspace_bytes_impl(n, nrhs, dt) || ((uintptr_t)ws % 256)) return DLA_ERR_WORKSPACE;
  constexpr int BOP = (KIND == KIND_LU) ? OP_SUB : OP_SUB_TN;  // the backward pass's one operation
  const int64_t nb = kNbMax, sb = kTriPair;
  const int64_t pairs = pairs_of(n);
  const int nblk = (int)pairs, last = nblk - 1;
  T* const wf = static_cast<T*>(ws);      // negated inverses, forward pass: pairs x (256 x 256)
  T* const wb = wf + pairs * sb * sb;     // negated inverses, backward pass (LU)
  T* const tf = wb + pairs * sb * sb;     // intermediates of the pairing: pairs x (128 x 128), forward
  T* const tb = tf + pairs * nb * nb;     // and backward
  T* const mf = tb + pairs * nb * nb;     // M of the forward pass: pairs x (256 x 512)
  T* const mb = mf + pairs * sb * 2 * sb; // M of the backward pass (Cholesky: its transpose, 512 x 256)
  T* const Y = mb + pairs * sb * 2 * sb;  // n x nrhs: Z and then the solution of the forward pass
  const int64_t ldy = y_ld(nrhs);
  T* const X = Y + n * ldy;               // n x nrhs: Z and then the solution of the backward pass
  auto rows_of = [&](int i) { return n - (int64_t)i * sb < sb ? n - (int64_t)i * sb : sb; };
  auto Nf = [&](int i) { return wf + (int64_t)i * sb * sb; };
  auto Nb = [&](int i) { return wb + (int64_t)i * sb * sb; };
  // Where the chain's launches run on the tiled GEMM (many right-hand sides) they use its 32 x 32 tiles: the
  // products stay skinny (k <= 512), and small tiles spread them over the compute units (N = 4000, 512
  // right-hand sides: 0.87 ms against 1.22 ms with 64 x 64 tiles; N = 8192, 1024: 4.33 against 4.63 ms).
  const GemmSchedule small = GemmSchedule{32, 32, 16, 4, 16, 16};
  const GemmSchedule sch = small;
  const GemmSchedule wide = GemmSchedule{64, 64, 16, 4, 32, 32};  // the 256 x 512 products of the pre-pass
  int rc;
  // ---- every target of a subtracting product that stands for a plain one starts at zero: the pre-pass's
  // targets lie in front of Y, the passes' own (Y and X) behind them
  {
    T* const from = prepare ? wf : Y;
    const int64_t count = (prepare ? block_elems(n) : 0) + (apply ? 2 * n * ldy : 0);
    hipLaunchKernelGGL(solve_zero_kernel<T>, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, from, count);
    if (launch_status(__func__) != DLA_SUCCESS) return DLA_ERR_HIP;
  }
  // with N = -W:  T = 0 - (off-diagonal block of the factor) * (N next to it) = block * W, then the
  // missing quarter of N = 0 - (the other N) * T = W * block * W
  auto pairing = [&](int pass, hipStream_t s) -> int {
    if (n <= nb) return DLA_SUCCESS;
    ProductList<T> first{small, OP_SUB}, second{small, OP_SUB};
    int r;
    for (int64_t p = 0; p < pairs; ++p) {
      const int64_t k0 = p * sb, b2 = n - k0 - nb < nb ? n - k0 - nb : nb;
      if (b2 <= 0) continue;  // a last block without a partner
      T* const W = (pass == 0 ? wf : wb) + p * sb * sb;
      T* const Tm = (pass == 0 ? tf : tb) + p * nb * nb;
      const T* const L21 = F + (k0 + nb) * lda + k0;  // b2 x 128
      const T* const U12 = F + k0 * lda + k0 + nb;    // 128 x b2
      if (pass == 0) r = first.add(L21, lda, W, sb, Tm, nb, b2, nb, nb, s);       // T = L21 W1
      else r = first.add(U12, lda, W + nb * sb + nb, sb, Tm, nb, nb, b2, b2, s);  // T = U12 V2
      if (r != DLA_SUCCESS) return r;
    }
    if ((r = first.flush(s)) != DLA_SUCCESS) return r;
    for (int64_t p = 0; p < pairs; ++p) {
      const int64_t k0 = p * sb, b2 = n - k0 - nb < nb ? n - k0 - nb : nb;
      if (b2 <= 0) continue;
      T* const W = (pass == 0 ? wf : wb) + p * sb * sb;
      const T* const Tm = (pass == 0 ? tf : tb) + p * nb * nb;
      if (pass == 0) r = second.add(W + nb * sb + nb, sb, Tm, nb, W + nb * sb, sb, b2, nb, b2, s);  // N21 = W2 T
      else r = second.add(W, sb, Tm, nb, W + nb, sb, nb, b2, nb, s);                                 // N12 = V1 T
      if (r != DLA_SUCCESS) return r;
    }
    return second.flush(s);
  };
  // M_i = 0 - N_i * (the factor's blocks beside diagonal block i that the look-back covers)
  auto look_back = [&](int pass, hipStream_t s) -> int {
    ProductList<T> list{wide, OP_SUB};
    int r = DLA_SUCCESS;
    if (pass == 0) {
      for (int i = 1; i < nblk && r == DLA_SUCCESS; ++i) {  // block columns i-2 (if any) and i-1 of block row i
        const int64_t c0 = (int64_t)(i >= 2 ? i - 2 : 0) * sb, kc = (int64_t)i * sb - c0;
        r = list.add(Nf(i), sb, F + (int64_t)i * sb * lda + c0, lda, mf + (int64_t)i * sb * 2 * sb, 2 * sb, rows_of(i), kc,
                     rows_of(i), s);
      }
    } else {
      for (int k = 0; k < last && r == DLA_SUCCESS; ++k) {  // block columns k+1 and k+2 (if any) of block row k
        const int64_t c0 = (int64_t)(k + 1) * sb, kc = (n < c0 + 2 * sb ? n : c0 + 2 * sb) - c0;
        if (KIND == KIND_LU)  // M_k = V_k [U_k,k+1  U_k,k+2]
          r = list.add(Nb(k), sb, F + (int64_t)k * sb * lda + c0, lda, mb + (int64_t)k * sb * 2 * sb, 2 * sb, sb, kc, sb, s);
        else  // M_k^T = [L_k+1,k ; L_k+2,k] W_k   (V_k = W_k^T and U_kj = L_jk^T)
          r = list.add(F + c0 * lda + (int64_t)k * sb, lda, Nf(k), sb, mb + (int64_t)k * sb * 2 * sb, sb, kc, sb, sb, s);
      }
    }
    return r != DLA_SUCCESS ? r : list.flush(s);
  };
  if (prepare) {
    if (KIND == KIND_LU)
      rc = launch_prepare_both<T, TRI_LOWER_UNIT, TRI_UPPER>(TriPrepareArgs<T>{F, lda, n, wf, T(-1)}, TriPrepareArgs<T>{F, lda, n, wb, T(-1)}, st);
    else
      rc = launch_prepare<T, TRI_LOWER>(TriPrepareArgs<T>{F, lda, n, wf, T(-1)}, st);
    if (rc != DLA_SUCCESS) return rc;
    if ((rc = pairing(0, st)) != DLA_SUCCESS) return rc;
    if (KIND == KIND_LU && (rc = pairing(1, st)) != DLA_SUCCESS) return rc;
    if ((rc = look_back(0, st)) != DLA_SUCCESS || (rc = look_back(1, st)) != DLA_SUCCESS) return rc;
  }
  if (!apply) return DLA_SUCCESS;
  // ---- the chain: one grouped launch per block step
  struct Part {
    const T *a, *b;
    T *c, *c2;
    int64_t la, lb, lc, lc2, M, K;
    int many;  // 1 for product (c): many blocks, the factor as its left operand
  };
  // While a launch of the chain is a few hundred to a few thousand 16 x 16 blocks, what matters is how soon its
  // longest product ends: the skinny kernel (one block per workgroup, k split over its waves; N = 4000, 64
  // right-hand sides 0.37 ms against 0.48 ms on 32 x 32 tiles with 128-deep slabs, 0.61 ms with 16-deep ones;
  // 256: 0.61 against 0.68 ms).  With more work per launch the tiled GEMM's reuse wins (N = 4000, 512: 0.98
  // against 0.87 ms; N = 8192, 256: 1.99 against 1.89 ms).
  const bool skinny = nrhs <= 128 || (nrhs <= 256 && n * nrhs <= 1200000);
  static_assert(2 * kTriPair <= kSkinnyMaxK, "the look-back product's depth");
  auto launch_parts = [&](int op, const Part* parts, int count) -> int {
    if (skinny) {
      SkinnyGroup<T> sg;
      int np = 0, wgs = 0, kmax = 0;
      double flops = 0.0;
      for (int q = 0; q < count; ++q) {
        const Part& P = parts[q];
        if (P.M <= 0 || P.K <= 0) continue;
        SkinnyPart<T>& sp = sg.part[np++];
        const int wide = (P.many && nrhs > 16 && P.K <= 256) ? 1 : 0;
        sp = SkinnyPart<T>{P.a, P.b, P.c, P.c2, P.la, P.lb, P.lc, P.lc2, (int)P.M, (int)nrhs, (int)P.K,
                           (int)((nrhs + (wide ? 31 : 15)) / (wide ? 32 : 16)), wgs, wide};
        wgs += skinny_workgroups(P.M, sp.tiles_n);
        kmax = P.K > kmax ? (int)P.K : kmax;
        flops += 2.0 * (double)P.M * (double)nrhs * (double)P.K;
      }
      if (np == 0) return DLA_SUCCESS;
      for (int q = np; q < kSkinnyMaxParts; ++q) sg.part[q] = sg.part[0];
      sg.nparts = np;
      return launch_skinny<T>(op == OP_SUB_TN, sg, wgs, kmax, flops, st);
    }
    GemmGroup<T> g;
    int np = 0, tiles = 0;
    double flops = 0.0;
    for (int q = 0; q < count; ++q) {
      const Part& P = parts[q];
      if (P.M <= 0 || P.K <= 0) continue;
      g.prob[np] = make_problem<T>(sch, op, P.a, P.la, P.b, P.lb, P.c, P.lc, P.M, nrhs, P.K, tiles);
      g.prob[np].C2 = P.c2;
      g.prob[np].ldc2 = P.lc2;
      tiles += problem_tiles(sch, op, g.prob[np]);
      flops += 2.0 * (double)P.M * (double)nrhs * (double)P.K;
      ++np;
    }
    if (np == 0) return DLA_SUCCESS;
    for (int q = np; q < kMaxGroup; ++q) g.prob[q] = g.prob[0];
    g.nprob = np;
    g.total_tiles = tiles;
    ProfileScope scope(PHASE_GEMM, flops, st);
    return launch_gemm<T>(sch, op, g, st);
  };
  // ---- forward.  Z_i and then Y_i live in rows i of Y; B is updated in place (part c).
  {
    Part head[2] = {{Nf(0), B, Y, nullptr, sb, ldb, ldy, 0, rows_of(0), rows_of(0)}, {}};
    if (nblk > 1) head[1] = Part{Nf(1), B + sb * ldb, Y + sb * ldy, nullptr, sb, ldb, ldy, 0, rows_of(1), rows_of(1)};
    if ((rc = launch_parts(OP_SUB, head, 2)) != DLA_SUCCESS) return rc;
  }
  for (int k = 0; k < last; ++k) {
    const int64_t k0 = (int64_t)k * sb;
    const int64_t c0 = (int64_t)(k >= 1 ? k - 1 : 0) * sb, kc = k0 + sb - c0;  // rows of Y that M_{k+1} multiplies
    const int64_t r3 = k0 + 3 * sb;                                            // first row of part (c)
    // (c) first: its workgroups wait longest for their operand (the factor, from HBM), so they are dispatched
    // first (N = 4000, 64 right-hand sides: 0.365 ms against 0.380 ms with (c) last)
    Part parts[3] = {
        {},
        {mf + (int64_t)(k + 1) * sb * 2 * sb, Y + c0 * ldy, Y + (k0 + sb) * ldy, nullptr, 2 * sb, ldy, ldy, 0, rows_of(k + 1), kc, 0},
        {}};
    if (r3 < n) parts[0] = Part{F + r3 * lda + k0, Y + k0 * ldy, B + r3 * ldb, nullptr, lda, ldy, ldb, 0, n - r3, sb, 1};
    if (k + 2 < nblk)
      parts[2] = Part{Nf(k + 2), B + (k0 + 2 * sb) * ldb, Y + (k0 + 2 * sb) * ldy, nullptr, sb, ldb, ldy, 0, rows_of(k + 2), rows_of(k + 2), 0};
    if ((rc = launch_parts(OP_SUB, parts, 3)) != DLA_SUCCESS) return rc;
  }
  // ---- backward.  Z_k and then X_k live in rows k of X (finished blocks are stored to B as well); Y is
  // updated in place (part c).  Cholesky: every left operand is read transposed (stored k x m).
  {
    const int64_t l0 = (int64_t)last * sb;
    Part head[2] = {{KIND == KIND_LU ? Nb(last) : Nf(last), Y + l0 * ldy, X + l0 * ldy, B + l0 * ldb, sb, ldy, ldy, ldb,
                     rows_of(last), rows_of(last)},
                    {}};
    if (last >= 1)
      head[1] = Part{KIND == KIND_LU ? Nb(last - 1) : Nf(last - 1), Y + (l0 - sb) * ldy, X + (l0 - sb) * ldy, nullptr, sb, ldy, ldy, 0, sb, sb};
    if ((rc = launch_parts(BOP, head, 2)) != DLA_SUCCESS) return rc;
  }
  for (int k = last; k >= 1; --k) {
    const int64_t k0 = (int64_t)k * sb;
    const int64_t kc = (n < k0 + 2 * sb ? n : k0 + 2 * sb) - k0;  // rows of X that M_{k-1} multiplies: blocks k, k+1
    const int64_t r1 = k0 - 2 * sb;                               // part (c) covers rows 0 .. r1
    const T* const m_prev = mb + (int64_t)(k - 1) * sb * 2 * sb;
    Part parts[3] = {
        {},
        {m_prev, X + k0 * ldy, X + (k0 - sb) * ldy, B + (k0 - sb) * ldb, KIND == KIND_LU ? 2 * sb : sb, ldy, ldy, ldb, sb, kc, 0},
        {}};
    if (r1 > 0) parts[0] = Part{KIND == KIND_LU ? F + k0 : F + k0 * lda, X + k0 * ldy, Y, nullptr, lda, ldy, ldy, 0, r1, rows_of(k), 1};
    if (k >= 2)
      parts[2] = Part{KIND == KIND_LU ? Nb(k - 2) : Nf(k - 2), Y + (k0 - 2 * sb) * ldy, X + (k0 - 2 * sb) * ldy, nullptr, sb, ldy, ldy, 0, sb, sb, 0};
    if ((rc = launch_parts(BOP, parts, 3)) != DLA_SUCCESS) return rc;
  }
  return DLA_SUCCESS;
}

template int solve_impl<double, KIND_LU>(const double*, int64_t, int64_t, double*, int64_t, int64_t, void*, size_t, hipStream_t, int);
template int solve_impl<float, KIND_LU>(const float*, int64_t, int64_t, float*, int64_t, int64_t, void*, size_t, hipStream_t, int);
template int solve_impl<double, KIND_CHOL>(const double*, int64_t, int64_t, double*, int64_t, int64_t, void*, size_t, hipStream_t, int);
template int solve_impl<float, KIND_CHOL>(const float*, int64_t, int64_t, float*, int64_t, int64_t, void*, size_t, hipStream_t, int);

}  // namespace dla
