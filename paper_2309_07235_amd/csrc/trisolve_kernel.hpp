// Solving with the factors (paper, Section "Linear Algebra Benchmarks": both decompositions are
// introduced as the way to solve systems of linear equations):  A X = B  becomes  L Y = B, U X = Y
// after lu_factor and  L Y = B, L^T X = Y  after cholesky_factor.  The host driver walks the
// triangular matrix in blocks of up to 128 rows; per block this kernel solves the block's own
// triangular system for all right-hand sides, and a tiled GEMM carries the solved rows into the
// rows that are still open.
//
// The kernel is the panel solve of the factorisations turned by 90 degrees: a wavefront owns 16
// right-hand sides (columns of B) as eight 16 x 16 accumulator blocks and runs the blocked
// forward substitution of head_solve on MFMA.  All four triangular matrices are brought to the
// one form that routine takes, lower triangular M' with  X' = M'^-1 P':
//   TRI_LOWER_UNIT   M' = L (unit diagonal implied; LU forward pass)
//   TRI_LOWER        M' = L (Cholesky forward pass)
//   TRI_UPPER        M' = J U J    with J the reversal of the block's rows (LU backward pass)
//   TRI_LOWER_TRANS  M' = J L^T J  (Cholesky backward pass; L^T is never formed in memory)
// and P' = B resp. J B.  A block shorter than a multiple of 16 is padded with the identity.
// head_solve wants the diagonal 16 x 16 sub-blocks inverted.  The inverses the factorisation made
// are gone with its workspace, so a pre-pass (tri_prepare_kernel, one workgroup per diagonal block,
// all blocks at once) stages every M', inverts its sub-blocks in registers, one 16-lane row per
// sub-block, and leaves the result in the solve's workspace; trisolve_kernel, which sits on the
// chain of the substitution, then only loads one contiguous run.
#pragma once
#include "head_kernel.hpp"

namespace dla {

enum TriMode { TRI_LOWER_UNIT = 0, TRI_LOWER = 1, TRI_UPPER = 2, TRI_LOWER_TRANS = 3 };
constexpr int kTriThreads = 256;

template <typename T>
struct TriSolveArgs {
  const T* M;   // the block as tri_prepare_kernel left it in the workspace
  T* B;         // the block's rows of the right-hand sides (b x nrhs), overwritten by the solution
  int64_t ldb;
  int b;        // 1 <= b <= kNbMax
  int nrhs;
};

template <typename T>
constexpr int trisolve_lds_bytes() {
  constexpr int nb = kNbMax / kIb;
  return (nb * (nb + 1) / 2) * kBlk * (int)sizeof(T);
}

// x = row i of the inverse of the lower-triangular matrix whose row i is a[0..i]; lane i of a
// 16-lane row owns row i.  UNIT: unit diagonal (a[i] ignored), else rdiag[k] = 1 / diagonal k.
template <typename T, bool UNIT>
__device__ inline void tri_inv16(const T (&a)[16], const T (&rdiag)[16], T (&x)[16], int i) {
#pragma unroll
  for (int j = 0; j < 16; ++j) x[j] = (j == i) ? T(1) : T(0);
  static_for<0, 16>([&](auto kc) {
    constexpr int k = decltype(kc)::value;
    if (!UNIT) {
      const T scale = (i == k) ? rdiag[k] : T(1);
      static_for<0, k + 1>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        x[j] *= scale;
      });
    }
    const T mult = (i > k) ? a[k] : T(0);
    static_for<0, k + 1>([&](auto jc) {
      constexpr int j = decltype(jc)::value;
      fnmac_bcast<k>(x[j], x[j], mult);  // x[j] -= a[i][k] * (row k of the inverse)[j]
    });
  });
}

// Pre-pass, one workgroup per diagonal block of the factor: stages M' of that block, inverts its
// diagonal sub-blocks, and writes the result (the layout head_solve reads) to the workspace.  It
// does not depend on the right-hand sides, so it runs once per call, all blocks in parallel,
// instead of on the chain of the substitution.
template <typename T>
struct TriPrepareArgs {
  const T* F;   // the factor (n x n, leading dimension lda)
  int64_t lda;
  int64_t n;
  T* out;       // one staged block of trisolve_lds_bytes<T>() bytes per diagonal block
};

template <typename T, int MODE>
__global__ void __launch_bounds__(kTriThreads) tri_prepare_kernel(const TriPrepareArgs<T> g) {
  constexpr int NB = kNbMax / kIb;
  constexpr int NTRI = NB * (NB + 1) / 2;
  constexpr bool REV = MODE == TRI_UPPER || MODE == TRI_LOWER_TRANS;
  constexpr bool UNIT = MODE == TRI_LOWER_UNIT;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  T* const tri = reinterpret_cast<T*>(smem_raw);

  const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l15 = lane & 15, l4 = lane >> 4;
  const int64_t k0 = (int64_t)blockIdx.x * kNbMax;
  const int b = (int)(g.n - k0 < kNbMax ? g.n - k0 : kNbMax);
  const int nblk = (b + kIb - 1) / kIb, bp = nblk * kIb;
  const int64_t lda = g.lda;
  const T* const D = g.F + k0 * lda + k0;
  auto orig = [&](int i) { return REV ? bp - 1 - i : i; };  // row of the block behind row i of M'

  // ---- stage M': sub-block (hi, lo), hi >= lo, at slot hi (hi + 1) / 2 + lo, element (rr, cc) at
  // rr * 17 + cc; one element per thread and sub-block.  Outside the block: the identity.
  // Every load is unconditional (indices clamped into the block, the value replaced afterwards) and
  // all of them are issued before the first LDS store: one round trip to memory for the whole block.
  {
    const int rr = tid >> 4, cc = tid & 15;
    T v[NTRI];
#pragma unroll
    for (int hi = 0; hi < NB; ++hi)
#pragma unroll
      for (int lo = 0; lo <= hi; ++lo) {
        if (hi < nblk) {  // uniform
          const int ii = orig(hi * kIb + rr), kk = orig(lo * kIb + cc);
          const int ic = ii < b ? ii : b - 1, kc = kk < b ? kk : b - 1;
          // lower forms read L[ii][kk] (ii >= kk); TRI_UPPER reads U[ii][kk] (ii <= kk after the
          // reversal); TRI_LOWER_TRANS reads (L^T)[ii][kk] = L[kk][ii]
          v[hi * (hi + 1) / 2 + lo] = (MODE == TRI_LOWER_TRANS) ? D[(int64_t)kc * lda + ic] : D[(int64_t)ic * lda + kc];
        }
      }
#pragma unroll
    for (int hi = 0; hi < NB; ++hi)
#pragma unroll
      for (int lo = 0; lo <= hi; ++lo) {
        if (hi < nblk) {
          const int i = hi * kIb + rr, k = lo * kIb + cc;
          const int ii = orig(i), kk = orig(k);
          T x = v[hi * (hi + 1) / 2 + lo];
          if (ii >= b || kk >= b) x = (ii == kk) ? T(1) : T(0);
          else if (UNIT && ii == kk) x = T(1);
          if (i < k) x = T(0);  // above the diagonal of a diagonal sub-block
          tri[(hi * (hi + 1) / 2 + lo) * kBlk + rr * (kIb + 1) + cc] = x;
        }
      }
  }
  __syncthreads();

  // ---- invert the diagonal sub-blocks in place: waves 0, 1, sub-block 4 * wave + l4
  if (wave < 2) {
    const int q = wave * 4 + l4;
    T* const d = tri + (q * (q + 1) / 2 + q) * kBlk + l15 * (kIb + 1);
    T a[16], rd[16], x[16];
    const bool on = q < nblk;
#pragma unroll
    for (int j = 0; j < 16; ++j) a[j] = on ? d[j] : (j == l15 ? T(1) : T(0));
    static_for<0, 16>([&](auto kc) {
      constexpr int k = decltype(kc)::value;
      rd[k] = UNIT ? T(1) : T(1) / row_bcast<k>(a[k]);
    });
    tri_inv16<T, UNIT>(a, rd, x, l15);
    if (on) {
#pragma unroll
      for (int j = 0; j < 16; ++j) d[j] = (j <= l15) ? x[j] : T(0);
    }
  }
  __syncthreads();

  // ---- out: the slots in use, as they sit in LDS (padding elements included: they are never read)
  T* const out = g.out + (int64_t)blockIdx.x * (NTRI * kBlk);
  const int used = (nblk * (nblk + 1) / 2) * kBlk;
  for (int e = tid; e < used; e += kTriThreads) out[e] = tri[e];
}

// REV: the block's rows are taken in reverse order (the backward passes).
template <typename T, bool REV>
__global__ void __launch_bounds__(kTriThreads) trisolve_kernel(const TriSolveArgs<T> g) {
  constexpr int NB = kNbMax / kIb;
  using acc_t = typename Mfma<T>::acc_t;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  T* const tri = reinterpret_cast<T*>(smem_raw);

  const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l15 = lane & 15, l4 = lane >> 4;
  const int b = g.b, nblk = (b + kIb - 1) / kIb, bp = nblk * kIb;
  const int64_t ldb = g.ldb;
  auto orig = [&](int i) { return REV ? bp - 1 - i : i; };  // row of the block behind row i of M'

  // ---- right-hand sides into the accumulators: register v of acc[s] is row 16 s + 4 l4 + v of P'
  const int slice0 = ((int)blockIdx.x * (kTriThreads / 64) + wave) * kIb;
  const bool job_on = slice0 < g.nrhs;
  const int t_valid = g.nrhs - slice0 < kIb ? g.nrhs - slice0 : kIb;
  const int t = slice0 + (l15 < t_valid ? l15 : t_valid - 1);
  acc_t acc[NB];
#pragma unroll
  for (int s = 0; s < NB; ++s) {
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int ii = orig(s * kIb + 4 * l4 + v);
      const bool in = job_on && s < nblk && ii < b;
      const T x = g.B[(int64_t)(in ? ii : 0) * ldb + (job_on ? t : 0)];
      acc[s][v] = in ? x : T(0);
    }
  }

  // ---- the prepared block: one contiguous run, two elements per load
  {
    struct alignas(2 * sizeof(T)) Pair { T lo, hi; };
    const int used2 = (nblk * (nblk + 1) / 2) * kBlk / 2;  // kBlk is even
    const Pair* const src = reinterpret_cast<const Pair*>(g.M);
    Pair* const dst = reinterpret_cast<Pair*>(tri);
    constexpr int MAX_IT = (NB * (NB + 1) / 2 * kBlk / 2 + kTriThreads - 1) / kTriThreads;
    Pair v[MAX_IT];
#pragma unroll
    for (int it = 0; it < MAX_IT; ++it) {
      const int e = tid + it * kTriThreads;
      v[it] = src[e < used2 ? e : used2 - 1];
    }
#pragma unroll
    for (int it = 0; it < MAX_IT; ++it) {
      const int e = tid + it * kTriThreads;
      if (e < used2) dst[e] = v[it];
    }
  }
  __syncthreads();
  if (!job_on) return;

  if (nblk == NB) head_solve<T, true>(tri, kIb + 1, 1, nblk, lane, acc);
  else head_solve<T, false>(tri, kIb + 1, 1, nblk, lane, acc);

  if (l15 < t_valid) {
#pragma unroll
    for (int s = 0; s < NB; ++s) {
      if (s < nblk) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int ii = orig(s * kIb + 4 * l4 + v);
          if (ii < b) g.B[(int64_t)ii * ldb + t] = acc[s][v];
        }
      }
    }
  }
}

}  // namespace dla
