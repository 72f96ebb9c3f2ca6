// Solving with the factors (paper, Section "Introduction": LU and Cholesky are named as the
// factorisations behind solving systems of linear equations):  A X = B  becomes  L Y = B, U X = Y
// after lu_factor and  L Y = B, L^T X = Y  after cholesky_factor.  The host driver walks the
// triangular matrix in blocks of rows.  The blocks' own triangular systems are taken off the chain
// of the substitution by inverting every diagonal block up front (this kernel: one workgroup per
// 128-row block, all blocks at once, independent of the right-hand sides), so that a step of the
// chain is small products on the tiled GEMM.  The host pairs the 128-row inverses into inverses of
// 256-row blocks (two more small products per pair, all pairs at once), which halves the steps of
// the chain, and asks for the negated inverses (unit = -1) because its chain subtracts.
//
// The inversion is the panel solve of the factorisations run on the identity: the block is brought
// to the form head_solve takes, lower triangular M' with 16 x 16 sub-blocks whose diagonal ones are
// inverted in registers (one 16-lane row per sub-block), and a wavefront then owns 16 columns of
// the identity as eight accumulator blocks and substitutes on MFMA.
//   TRI_LOWER_UNIT   M' = L (unit diagonal implied; LU forward pass)
//   TRI_LOWER        M' = L (Cholesky forward pass)
//   TRI_UPPER        M' = J U J    with J the reversal of the block's rows (LU backward pass)
//   TRI_LOWER_TRANS  M' = J L^T J  (the inverse of L^T; the host driver reads the inverse of L transposed
//                    instead and does not use this mode)
// The result is stored un-reversed, W = J M'^-1 J.  A block shorter than a multiple of 16 is padded
// with the identity.
#pragma once
#include "head_kernel.hpp"

namespace dla {

enum TriMode { TRI_LOWER_UNIT = 0, TRI_LOWER = 1, TRI_UPPER = 2, TRI_LOWER_TRANS = 3 };
constexpr int kTriThreads = 256;

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

// One workgroup per diagonal block of the factor.  Two consecutive blocks share a 256 x 256 area
// of the output (row stride 256): block 2p at its top left, block 2p + 1 at its bottom right; the
// host fills in the off-diagonal quarter that makes the area the inverse of the 256-row block.
constexpr int kTriPair = 2 * kNbMax;
template <typename T>
struct TriPrepareArgs {
  const T* F;   // the factor (n x n, leading dimension lda)
  int64_t lda;
  int64_t n;
  T* out;       // one kTriPair x kTriPair area per pair of diagonal blocks
  T unit;       // 1: the inverses themselves; -1: the negated inverses (the substitution runs on -I)
};

// The work of one workgroup: diagonal block `block` of g's factor.
template <typename T, int MODE>
__device__ __forceinline__ void tri_prepare_block(const TriPrepareArgs<T>& g, const int block) {
  constexpr int NB = kNbMax / kIb;
  constexpr int NTRI = NB * (NB + 1) / 2;
  constexpr bool REV = MODE == TRI_UPPER || MODE == TRI_LOWER_TRANS;
  constexpr bool UNIT = MODE == TRI_LOWER_UNIT;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  T* const tri = reinterpret_cast<T*>(smem_raw);

  const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l15 = lane & 15, l4 = lane >> 4;
  const int64_t k0 = (int64_t)block * kNbMax;
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

  // ---- the block's inverse: the substitution run on the identity, 16 columns per wave and pass.
  // out holds W = M^-1 for the block in its own (un-reversed) index space, row-major, so that the
  // solve itself is the plain product W * B; what lies outside the b x b block is never read.
  using acc_t = typename Mfma<T>::acc_t;
  T* const out = g.out + (int64_t)(block >> 1) * (kTriPair * kTriPair) + (block & 1) * (kNbMax * kTriPair + kNbMax);
  for (int pass = 0; pass < NB / (kTriThreads / 64); ++pass) {
    const int slice = pass * (kTriThreads / 64) + wave;
    if (slice < nblk) {  // uniform per wave
      acc_t acc[NB];
#pragma unroll
      for (int s = 0; s < NB; ++s)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[s][v] = (s * kIb + 4 * l4 + v == slice * kIb + l15) ? g.unit : T(0);
      if (nblk == NB) head_solve<T, true>(tri, kIb + 1, 1, nblk, lane, acc);
      else head_solve<T, false>(tri, kIb + 1, 1, nblk, lane, acc);
      const int cc = orig(slice * kIb + l15);
#pragma unroll
      for (int s = 0; s < NB; ++s) {
        if (s < nblk) {
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int rr = orig(s * kIb + 4 * l4 + v);
            if (rr < b && cc < b) out[rr * kTriPair + cc] = acc[s][v];
          }
        }
      }
    }
  }
}

template <typename T, int MODE>
__global__ void __launch_bounds__(kTriThreads) tri_prepare_kernel(const TriPrepareArgs<T> g) {
  tri_prepare_block<T, MODE>(g, (int)blockIdx.x);
}

// Two sets of inverses of the same factor in one launch (they are independent): the first half of the
// grid works on ga in MODE_A, the second half on gb in MODE_B.
template <typename T, int MODE_A, int MODE_B>
__global__ void __launch_bounds__(kTriThreads) tri_prepare_both_kernel(const TriPrepareArgs<T> ga, const TriPrepareArgs<T> gb) {
  const int half = (int)(gridDim.x >> 1);
  if ((int)blockIdx.x < half) tri_prepare_block<T, MODE_A>(ga, (int)blockIdx.x);
  else tri_prepare_block<T, MODE_B>(gb, (int)blockIdx.x - half);
}

}  // namespace dla
