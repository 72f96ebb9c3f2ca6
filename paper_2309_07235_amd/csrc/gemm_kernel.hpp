// LDS-tiled MFMA GEMM for gfx950, the building block of 3mm (paper, 3mm_basic
// listing: three products with split y/x axes), of the LU trailing update
// A22 -= L21*U12 and of the Cholesky trailing update lower(A22) -= L21*L21^T.
//
// One workgroup computes a TM x TN macro-tile of C (the paper's y/x split
// factors); its waves are laid out WAVES_M x WAVES_N and each accumulates a
// WM x WN sub-tile in registers as (WM/16) x (WN/16) MFMA blocks.  The k axis is
// walked in slabs of TK staged through double-buffered LDS: while slab s is
// being multiplied, slab s+1 is in flight from global memory into registers,
// and is written to the other LDS buffer before the single barrier per slab.
//
// LDS layouts.  A rows keep k contiguous with an odd row stride (TK+1): the
// 16 lanes that read one fragment column then hit 16 distinct bank pairs.
// B (k x n) keeps n contiguous: a fragment row is one contiguous 128-byte run.
// For the A*B^T forms the right operand is stored like A.
#pragma once
#include "dla_common.hpp"

namespace dla {

enum GemmOp { OP_ASSIGN = 0, OP_SUB = 1, OP_SUB_NT_LOWER = 2, OP_SUB_NT = 3 };

template <typename T>
struct GemmProblem {
  const T* A;
  const T* B;
  T* C;
  int64_t lda, ldb, ldc;
  int M, N, K;
  int tiles_m, tiles_n;
  int tile_begin;  // first logical tile id of this problem inside the group
};

template <typename T>
struct GemmGroup {
  GemmProblem<T> prob[2];
  int nprob;
  int total_tiles;
};

template <int TM, int TN, int TK, int WM, int WN, bool BT, int ESZ>
struct GemmLds {
  static constexpr int SA = TK + 1;
  static constexpr int SB = BT ? TK + 1 : TN;
  static constexpr int A_ELEMS = TM * SA;
  static constexpr int B_ELEMS_RAW = BT ? TN * SB : TK * SB;
  // keep every buffer 16-byte aligned
  static constexpr int ALIGN_E = 16 / ESZ;
  static constexpr int A_PAD = (A_ELEMS + ALIGN_E - 1) / ALIGN_E * ALIGN_E;
  static constexpr int B_PAD = (B_ELEMS_RAW + ALIGN_E - 1) / ALIGN_E * ALIGN_E;
  static constexpr int STAGE = A_PAD + B_PAD;
  static constexpr int BYTES = 2 * STAGE * ESZ;
};

// Global -> register load of a ROWS x TK tile whose k axis is contiguous in
// memory (row r at base + r*ld).  Each thread takes pairs of k-neighbours.
template <typename T, int ROWS, int TK, int NT>
struct RowTileLoader {
  static constexpr int VPR = TK / 2;
  static constexpr int TOTAL = ROWS * VPR;
  static constexpr int ITER = (TOTAL + NT - 1) / NT;
  using vec2_t = typename Mfma<T>::vec2_t;
  T r[ITER][2];

  __device__ inline void load_full(const T* __restrict__ base, int64_t ld, int tid) {
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      const int idx = tid + it * NT;
      if (TOTAL % NT == 0 || idx < TOTAL) {
        const int row = idx / VPR, c2 = idx % VPR;
        const T* p = base + (int64_t)row * ld + 2 * c2;
        r[it][0] = p[0];
        r[it][1] = p[1];
      }
    }
  }
  // Edge tiles: every load is issued unconditionally from an address clamped into the valid
  // part (rows_valid, k_valid >= 1) and zeroed afterwards, so no load waits behind a branch.
  __device__ inline void load_edge(const T* __restrict__ base, int64_t ld, int tid, int rows_valid, int k_valid) {
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      const int idx = tid + it * NT;
      if (TOTAL % NT == 0 || idx < TOTAL) {
        const int row = idx / VPR, c0 = 2 * (idx % VPR), c1 = c0 + 1;
        const T* p = base + (int64_t)(row < rows_valid ? row : rows_valid - 1) * ld;
        const T x0 = p[c0 < k_valid ? c0 : k_valid - 1], x1 = p[c1 < k_valid ? c1 : k_valid - 1];
        r[it][0] = (row < rows_valid && c0 < k_valid) ? x0 : T(0);
        r[it][1] = (row < rows_valid && c1 < k_valid) ? x1 : T(0);
      }
    }
  }
  template <bool NEGATE, int STRIDE>
  __device__ inline void store(T* __restrict__ s, int tid) const {
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      const int idx = tid + it * NT;
      if (TOTAL % NT == 0 || idx < TOTAL) {
        const int row = idx / VPR, c2 = idx % VPR;
        s[row * STRIDE + 2 * c2] = NEGATE ? -r[it][0] : r[it][0];
        s[row * STRIDE + 2 * c2 + 1] = NEGATE ? -r[it][1] : r[it][1];
      }
    }
  }
};

// Global -> register load of a TK x COLS tile of a row-major k x n operand
// (row k at base + k*ld, n contiguous).
template <typename T, int TK, int COLS, int NT>
struct ColTileLoader {
  static constexpr int VPR = COLS / 2;
  static constexpr int TOTAL = TK * VPR;
  static constexpr int ITER = (TOTAL + NT - 1) / NT;
  using vec2_t = typename Mfma<T>::vec2_t;
  T r[ITER][2];

  __device__ inline void load_full(const T* __restrict__ base, int64_t ld, int tid) {
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      const int idx = tid + it * NT;
      if (TOTAL % NT == 0 || idx < TOTAL) {
        const int kr = idx / VPR, c2 = idx % VPR;
        const T* p = base + (int64_t)kr * ld + 2 * c2;
        r[it][0] = p[0];
        r[it][1] = p[1];
      }
    }
  }
  __device__ inline void load_edge(const T* __restrict__ base, int64_t ld, int tid, int k_valid, int cols_valid) {
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      const int idx = tid + it * NT;
      if (TOTAL % NT == 0 || idx < TOTAL) {
        const int kr = idx / VPR, c0 = 2 * (idx % VPR), c1 = c0 + 1;
        const T* p = base + (int64_t)(kr < k_valid ? kr : k_valid - 1) * ld;
        const T x0 = p[c0 < cols_valid ? c0 : cols_valid - 1], x1 = p[c1 < cols_valid ? c1 : cols_valid - 1];
        r[it][0] = (kr < k_valid && c0 < cols_valid) ? x0 : T(0);
        r[it][1] = (kr < k_valid && c1 < cols_valid) ? x1 : T(0);
      }
    }
  }
  template <int STRIDE>
  __device__ inline void store(T* __restrict__ s, int tid) const {
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      const int idx = tid + it * NT;
      if (TOTAL % NT == 0 || idx < TOTAL) {
        const int kr = idx / VPR, c2 = idx % VPR;
        s[kr * STRIDE + 2 * c2] = r[it][0];
        s[kr * STRIDE + 2 * c2 + 1] = r[it][1];
      }
    }
  }
};

template <typename T, int TM, int TN, int TK, int WM, int WN, int UK, int OP>
__global__ void __launch_bounds__((TM / WM) * (TN / WN) * 64)
gemm_kernel(const GemmGroup<T> g) {
  static_assert(TM % WM == 0 && TN % WN == 0 && WM % 16 == 0 && WN % 16 == 0, "tile shape");
  static_assert(TK % 4 == 0 && TK % 2 == 0, "k slab");
  constexpr int WAVES_N = TN / WN;
  constexpr int NW = (TM / WM) * WAVES_N;
  constexpr int NT = NW * 64;
  constexpr int FM = WM / 16, FN = WN / 16, KSTEPS = TK / 4;
  constexpr bool BT = (OP == OP_SUB_NT_LOWER || OP == OP_SUB_NT);
  constexpr bool LOWER = (OP == OP_SUB_NT_LOWER);
  constexpr bool SUB = (OP != OP_ASSIGN);
  using L = GemmLds<TM, TN, TK, WM, WN, BT, (int)sizeof(T)>;
  using acc_t = typename Mfma<T>::acc_t;

  extern __shared__ __align__(16) unsigned char smem_raw[];
  T* const smem = reinterpret_cast<T*>(smem_raw);

  // ---- which tile ----------------------------------------------------------------
  const int logical = xcd_contiguous_id((int)blockIdx.x, g.total_tiles);
  const int pi = (g.nprob > 1 && logical >= g.prob[1].tile_begin) ? 1 : 0;
  const GemmProblem<T>& P = g.prob[pi];
  const int local = logical - P.tile_begin;
  int ti, tj;
  if (LOWER && TM == TN) {  // lower-triangular tile set, row by row
    int i = (int)((sqrtf(8.0f * (float)local + 1.0f) - 1.0f) * 0.5f);
    while ((int64_t)i * (i + 1) / 2 > local) --i;
    while ((int64_t)(i + 1) * (i + 2) / 2 <= local) ++i;
    ti = i;
    tj = local - i * (i + 1) / 2;
  } else {
    ti = local / P.tiles_n;
    tj = local % P.tiles_n;
  }
  const int m0 = ti * TM, n0 = tj * TN;
  if (LOWER && n0 >= m0 + TM) return;  // tile strictly above the diagonal (only when TM != TN)

  const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int M = P.M, N = P.N, K = P.K;
  const int64_t lda = P.lda, ldb = P.ldb, ldc = P.ldc;
  const bool full_mn = (m0 + TM <= M) && (n0 + TN <= N);
  const int l15 = lane & 15, l4 = lane >> 4;

  // ---- accumulators: C tile for the subtracting forms, zero otherwise ------------
  acc_t acc[FM][FN];
  T* const Cw = P.C + (int64_t)(m0 + wm0) * ldc + (n0 + wn0);
  if (SUB) {
    if (full_mn) {  // interior tile: constant offsets from one base pointer
#pragma unroll
      for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b)
#pragma unroll
          for (int v = 0; v < 4; ++v)
            acc[a][b][v] = Cw[(int64_t)(a * 16 + Mfma<T>::row_of(v, lane)) * ldc + b * 16 + l15];
    } else {  // edge tile: clamped address, masked value, so the preload never branches per element
#pragma unroll
      for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int r = a * 16 + Mfma<T>::row_of(v, lane), c = b * 16 + l15;
            const bool in = (m0 + wm0 + r < M) && (n0 + wn0 + c < N);
            const int rc = (m0 + wm0 + r < M) ? r : M - 1 - m0 - wm0;
            const int cc = (n0 + wn0 + c < N) ? c : N - 1 - n0 - wn0;
            const T x = Cw[(int64_t)rc * ldc + cc];
            acc[a][b][v] = in ? x : T(0);
          }
    }
  } else {
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
      for (int b = 0; b < FN; ++b) acc[a][b] = acc_t{0, 0, 0, 0};
  }

  // ---- main loop -----------------------------------------------------------------
  RowTileLoader<T, TM, TK, NT> la;
  RowTileLoader<T, TN, TK, NT> lbt;   // right operand when it is n x k (BT)
  ColTileLoader<T, TK, TN, NT> lbn;   // right operand when it is k x n
  const T* const Ag = P.A + (int64_t)m0 * lda;
  const T* const Bg = BT ? P.B + (int64_t)n0 * ldb : P.B + n0;
  const int nslab = (K + TK - 1) / TK;

  auto fetch = [&](int s) {
    const int k0 = s * TK;
    const bool full = full_mn && (k0 + TK <= K);
    if (full) {
      la.load_full(Ag + k0, lda, tid);
      if (BT) lbt.load_full(Bg + k0, ldb, tid);
      else lbn.load_full(Bg + (int64_t)k0 * ldb, ldb, tid);
    } else {
      la.load_edge(Ag + k0, lda, tid, M - m0, K - k0);
      if (BT) lbt.load_edge(Bg + k0, ldb, tid, N - n0, K - k0);
      else lbn.load_edge(Bg + (int64_t)k0 * ldb, ldb, tid, K - k0, N - n0);
    }
  };
  auto stash = [&](int buf) {
    T* sa = smem + buf * L::STAGE;
    T* sb = sa + L::A_PAD;
    la.template store<SUB, L::SA>(sa, tid);  // subtracting forms multiply by -A
    if (BT) lbt.template store<false, L::SB>(sb, tid);
    else lbn.template store<L::SB>(sb, tid);
  };

  if (nslab > 0) {
    fetch(0);
    stash(0);
  }
  lds_barrier();

  for (int s = 0; s < nslab; ++s) {
    const bool more = (s + 1 < nslab);
    if (more) fetch(s + 1);
    const T* sa = smem + (s & 1) * L::STAGE;
    const T* sb = sa + L::A_PAD;
    const T* pa = sa + (wm0 + l15) * L::SA + l4;
    const T* pb = BT ? sb + (wn0 + l15) * L::SB + l4 : sb + l4 * L::SB + wn0 + l15;
#pragma unroll UK
    for (int kk = 0; kk < KSTEPS; ++kk) {
      T fa[FM], fb[FN];
#pragma unroll
      for (int a = 0; a < FM; ++a) fa[a] = pa[a * 16 * L::SA + kk * 4];
#pragma unroll
      for (int b = 0; b < FN; ++b) fb[b] = BT ? pb[b * 16 * L::SB + kk * 4] : pb[kk * 4 * L::SB + b * 16];
#pragma unroll
      for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b) acc[a][b] = Mfma<T>::mma(fa[a], fb[b], acc[a][b]);
    }
    if (more) stash((s + 1) & 1);
    lds_barrier();
  }

  // ---- store ---------------------------------------------------------------------
#pragma unroll
  for (int a = 0; a < FM; ++a)
#pragma unroll
    for (int b = 0; b < FN; ++b)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int r = a * 16 + Mfma<T>::row_of(v, lane), c = b * 16 + l15;
        if (full_mn || (m0 + wm0 + r < M && n0 + wn0 + c < N)) Cw[(int64_t)r * ldc + c] = acc[a][b][v];
      }
}

}  // namespace dla
