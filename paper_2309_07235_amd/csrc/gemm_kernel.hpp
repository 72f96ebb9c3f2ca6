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
// For the A*B^T forms the right operand is stored like A; for the A^T*B form the left operand
// (k x m in memory) is stored like B.
#pragma once
#include <type_traits>
#include "dla_common.hpp"

namespace dla {

// OP_SUB_TN: C -= A^T * B with A stored k x m (the Cholesky backward substitution multiplies by L^T
// without forming it); instantiated for the two small macro-tiles only.
enum GemmOp { OP_ASSIGN = 0, OP_SUB = 1, OP_SUB_NT_LOWER = 2, OP_SUB_NT = 3, OP_SUB_TN = 4 };

template <typename T>
struct GemmProblem {
  const T* A;
  const T* B;
  T* C;
  int64_t lda, ldb, ldc;
  int M, N, K;
  int tiles_m, tiles_n;
  int tile_begin;  // first logical tile id of this problem inside the group
  T* C2;           // optional second destination of the result (same shape, leading dimension ldc2), or null
  int64_t ldc2;
};

constexpr int kMaxGroup = 16;  // products one launch can carry

template <typename T>
struct GemmGroup {
  GemmProblem<T> prob[kMaxGroup];
  int nprob;
  int total_tiles;
};

template <int TM, int TN, int TK, int WM, int WN, bool BT, int ESZ, bool AT = false>
struct GemmLds {
  static constexpr int SA = AT ? TM : TK + 1;
  static constexpr int SB = BT ? TK + 1 : TN;
  static constexpr int A_ELEMS = AT ? TK * SA : TM * SA;
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
// Row pointers are set up once per tile (rows past the edge are clamped into the
// matrix and masked), so a slab load is a handful of loads at constant offsets.
template <typename T, int ROWS, int TK, int NT>
struct RowTileLoader {
  static constexpr int VPR = TK / 2;
  static constexpr int TOTAL = ROWS * VPR;
  static constexpr int ITER = (TOTAL + NT - 1) / NT;
  const T* p[ITER];  // element (row, 2*c2) of slab 0
  bool ok[ITER];     // row inside the matrix
  T r[ITER][2];

  __device__ __forceinline__ void init(const T* __restrict__ base, int64_t ld, int tid, int rows_valid) {
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      const int idx = tid + it * NT;
      const int row = idx / VPR, c2 = idx % VPR;
      const bool in = (TOTAL % NT == 0 || idx < TOTAL) && row < rows_valid;
      ok[it] = in;
      p[it] = base + (int64_t)(in ? row : rows_valid - 1) * ld + 2 * c2;
    }
  }
  // full slab of an interior tile
  __device__ __forceinline__ void load_full(int k0) {
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      r[it][0] = p[it][k0];
      r[it][1] = p[it][k0 + 1];
    }
  }
  // any slab of an edge tile, or the last (partial) slab: k_valid = K - k0 >= 1.
  // Loads stay unconditional (clamped k) and are NOT touched here: the mask is applied when the
  // registers are written to LDS, so the loads stay in flight while the previous slab is multiplied.
  __device__ __forceinline__ void load_edge(int k0, int k_valid, int tid) {
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      const int c0 = 2 * ((tid + it * NT) % VPR), c1 = c0 + 1;
      r[it][0] = p[it][k0 + (c0 < k_valid ? 0 : k_valid - 1 - c0)];
      r[it][1] = p[it][k0 + (c1 < k_valid ? 1 : k_valid - 1 - c0)];
    }
  }
  // MASK: zero what lies outside the matrix (edge tile or partial slab)
  template <bool NEGATE, int STRIDE, bool MASK>
  __device__ __forceinline__ void store(T* __restrict__ s, int tid, int k_valid) const {
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      const int idx = tid + it * NT;
      if (TOTAL % NT == 0 || idx < TOTAL) {
        const int row = idx / VPR, c2 = idx % VPR;
        T x0 = r[it][0], x1 = r[it][1];
        if (MASK) {
          x0 = (ok[it] && 2 * c2 < k_valid) ? x0 : T(0);
          x1 = (ok[it] && 2 * c2 + 1 < k_valid) ? x1 : T(0);
        }
        s[row * STRIDE + 2 * c2] = NEGATE ? -x0 : x0;
        s[row * STRIDE + 2 * c2 + 1] = NEGATE ? -x1 : x1;
      }
    }
  }
};

// Global -> register load of a TK x COLS tile of a row-major k x n operand
// (row k at base + k*ld, n contiguous).  Column offsets are clamped and masked once per tile.
template <typename T, int TK, int COLS, int NT>
struct ColTileLoader {
  static constexpr int VPR = COLS / 2;
  static constexpr int TOTAL = TK * VPR;
  static constexpr int ITER = (TOTAL + NT - 1) / NT;
  const T* base;
  int64_t ld;
  int c0[ITER], c1[ITER];    // clamped column offsets
  bool ok0[ITER], ok1[ITER];
  // a ragged tile with at least two valid columns: start of an in-bounds pair of neighbours that holds this
  // thread's valid columns, and whether its first column sits in the second place of that pair
  int cp[ITER];
  bool sh[ITER];
  T r[ITER][2];

  __device__ __forceinline__ void init(const T* __restrict__ b, int64_t ld_, int tid, int cols_valid) {
    base = b;
    ld = ld_;
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      const int idx = tid + it * NT;
      const int c = 2 * (idx % VPR);
      const bool in = (TOTAL % NT == 0 || idx < TOTAL);
      ok0[it] = in && c < cols_valid;
      ok1[it] = in && c + 1 < cols_valid;
      c0[it] = ok0[it] ? c : cols_valid - 1;
      c1[it] = ok1[it] ? c + 1 : cols_valid - 1;
      cp[it] = ok1[it] ? c : (cols_valid >= 2 ? cols_valid - 2 : 0);
      sh[it] = ok0[it] && !ok1[it];  // c is the last valid column: the pair starts one column before it
    }
  }
  // full slab of a ragged tile (cols_valid >= 2): same loads as an interior tile, at the in-bounds pairs
  __device__ __forceinline__ void load_ragged(int k0, int tid) {
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      const int kr = row_of(tid + it * NT);
      const T* q = base + (int64_t)(k0 + kr) * ld + cp[it];
      r[it][0] = q[0];
      r[it][1] = q[1];
    }
  }
  // threads beyond the tile (a tile smaller than the workgroup) re-read its last row
  static __device__ __forceinline__ int row_of(int idx) {
    const int kr = idx / VPR;
    return (TOTAL % NT == 0 || kr < TK) ? kr : TK - 1;
  }
  __device__ __forceinline__ void load_full(int k0, int tid) {
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      const int kr = row_of(tid + it * NT);
      const T* q = base + (int64_t)(k0 + kr) * ld + 2 * ((tid + it * NT) % VPR);
      r[it][0] = q[0];
      r[it][1] = q[1];
    }
  }
  __device__ __forceinline__ void load_edge(int k0, int k_valid, int tid) {
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      const int kr = (tid + it * NT) / VPR;
      const T* q = base + (int64_t)(k0 + (kr < k_valid ? kr : k_valid - 1)) * ld;
      r[it][0] = q[c0[it]];
      r[it][1] = q[c1[it]];
    }
  }
  // PAIRS: the registers were filled by load_ragged
  template <int STRIDE, bool MASK, bool NEGATE = false, bool PAIRS = false>
  __device__ __forceinline__ void store(T* __restrict__ s, int tid, int k_valid) const {
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      const int idx = tid + it * NT;
      if (TOTAL % NT == 0 || idx < TOTAL) {
        const int kr = idx / VPR, c2 = idx % VPR;
        T x0 = (PAIRS && sh[it]) ? r[it][1] : r[it][0], x1 = r[it][1];
        if (MASK) {
          x0 = (ok0[it] && kr < k_valid) ? x0 : T(0);
          x1 = (ok1[it] && kr < k_valid) ? x1 : T(0);
        }
        s[kr * STRIDE + 2 * c2] = NEGATE ? -x0 : x0;
        s[kr * STRIDE + 2 * c2 + 1] = NEGATE ? -x1 : x1;
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
  constexpr bool AT = (OP == OP_SUB_TN);
  using L = GemmLds<TM, TN, TK, WM, WN, BT, (int)sizeof(T), AT>;
  using acc_t = typename Mfma<T>::acc_t;

  extern __shared__ __align__(16) unsigned char smem_raw[];
  T* const smem = reinterpret_cast<T*>(smem_raw);

  // ---- which tile ----------------------------------------------------------------
  const int logical = xcd_contiguous_id((int)blockIdx.x, g.total_tiles);
  int pi = 0;
#pragma unroll
  for (int q = 1; q < kMaxGroup; ++q)
    if (q < g.nprob && logical >= g.prob[q].tile_begin) pi = q;
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
  ColTileLoader<T, TK, TM, NT> lat;   // left operand when it is k x m (AT)
  RowTileLoader<T, TN, TK, NT> lbt;   // right operand when it is n x k (BT)
  ColTileLoader<T, TK, TN, NT> lbn;   // right operand when it is k x n
  const T* const Ag = AT ? P.A + m0 : P.A + (int64_t)m0 * lda;
  const T* const Bg = BT ? P.B + (int64_t)n0 * ldb : P.B + n0;
  const int nslab = (K + TK - 1) / TK;

  if (AT) lat.init(Ag, lda, tid, M - m0);
  else la.init(Ag, lda, tid, M - m0);
  if (BT) lbt.init(Bg, ldb, tid, N - n0);
  else lbn.init(Bg, ldb, tid, N - n0);
  // Three copies of the pipeline, chosen per slab.  Interior slabs (whole tile inside the matrix, whole
  // slab inside K) load at constant offsets and store unmasked.  Whole slabs of a ragged tile take the
  // same loads at offsets that stay inside the matrix (rows clamped once per tile, columns as in-bounds
  // pairs) and a masked store.  The last, partial slab takes loads clamped per element.  Kept as
  // separate loops so that the fast ones stay free of per-element address arithmetic.
  auto fetch = [&](auto kind, int s) __attribute__((always_inline)) {
    const int k0 = s * TK;
    constexpr int KIND_OF_SLAB = decltype(kind)::value;
    if constexpr (KIND_OF_SLAB == 0) {
      if (AT) lat.load_full(k0, tid);
      else la.load_full(k0);
      if (BT) lbt.load_full(k0);
      else lbn.load_full(k0, tid);
    } else if constexpr (KIND_OF_SLAB == 1) {
      if (AT) lat.load_ragged(k0, tid);
      else la.load_full(k0);
      if (BT) lbt.load_full(k0);
      else lbn.load_ragged(k0, tid);
    } else {
      if (AT) lat.load_edge(k0, K - k0, tid);
      else la.load_edge(k0, K - k0, tid);
      if (BT) lbt.load_edge(k0, K - k0, tid);
      else lbn.load_edge(k0, K - k0, tid);
    }
  };
  auto stash = [&](auto kind, int buf, int s) __attribute__((always_inline)) {  // s: the slab that sits in the registers
    constexpr bool E = decltype(kind)::value != 0;  // masked
    constexpr bool P = decltype(kind)::value == 1;  // column pairs of a ragged tile
    T* sa = smem + buf * L::STAGE;
    T* sb = sa + L::A_PAD;
    const int kv = K - s * TK;
    if (AT) lat.template store<L::SA, E, SUB, P>(sa, tid, kv);
    else la.template store<SUB, L::SA, E>(sa, tid, kv);  // subtracting forms multiply by -A
    if (BT) lbt.template store<false, L::SB, E>(sb, tid, kv);
    else lbn.template store<L::SB, E, false, P>(sb, tid, kv);
  };
  // iterations [s0, s1): multiply slab s while slab s + 1 (when there is one) is fetched as slabs of kind `edge`
  auto slabs = [&](auto edge, int s0, int s1) __attribute__((always_inline)) {
    for (int s = s0; s < s1; ++s) {
      const bool more = decltype(edge)::value != 2 || (s + 1 < nslab);
      if (more) fetch(edge, s + 1);
      const T* sa = smem + (s & 1) * L::STAGE;
      const T* sb = sa + L::A_PAD;
      const T* pa = AT ? sa + l4 * L::SA + wm0 + l15 : sa + (wm0 + l15) * L::SA + l4;
      const T* pb = BT ? sb + (wn0 + l15) * L::SB + l4 : sb + l4 * L::SB + wn0 + l15;
#pragma unroll UK
      for (int kk = 0; kk < KSTEPS; ++kk) {
        T fa[FM], fb[FN];
#pragma unroll
        for (int a = 0; a < FM; ++a) fa[a] = AT ? pa[kk * 4 * L::SA + a * 16] : pa[a * 16 * L::SA + kk * 4];
#pragma unroll
        for (int b = 0; b < FN; ++b) fb[b] = BT ? pb[b * 16 * L::SB + kk * 4] : pb[kk * 4 * L::SB + b * 16];
#pragma unroll
        for (int a = 0; a < FM; ++a)
#pragma unroll
          for (int b = 0; b < FN; ++b) acc[a][b] = Mfma<T>::mma(fa[a], fb[b], acc[a][b]);
      }
      if (more) stash(edge, (s + 1) & 1, s + 1);
      lds_barrier();
    }
  };
  using interior_t = std::integral_constant<int, 0>;
  using ragged_t = std::integral_constant<int, 1>;
  using edge_t = std::integral_constant<int, 2>;
  // a ragged tile can load whole slabs pairwise when its operands with contiguous columns have two valid ones
  const bool pairs_ok = (!AT || M - m0 >= 2) && (BT || N - n0 >= 2);
  const int nfull = (full_mn || pairs_ok) ? K / TK : 0;  // leading slabs that are whole

  if (nfull > 0) {
    if (full_mn) {
      fetch(interior_t{}, 0);
      stash(interior_t{}, 0, 0);
    } else {
      fetch(ragged_t{}, 0);
      stash(ragged_t{}, 0, 0);
    }
  } else if (nslab > 0) {
    fetch(edge_t{}, 0);
    stash(edge_t{}, 0, 0);
  }
  lds_barrier();
  const int split = nfull > 0 ? nfull - 1 : 0;  // iterations below it prefetch a whole slab
  if (full_mn) slabs(interior_t{}, 0, split);
  else slabs(ragged_t{}, 0, split);
  slabs(edge_t{}, split, nslab);

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
  if (P.C2) {  // uniform: a copy of the result for a consumer that must not see later in-place changes
    T* const Cw2 = P.C2 + (int64_t)(m0 + wm0) * P.ldc2 + (n0 + wn0);
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
      for (int b = 0; b < FN; ++b)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int r = a * 16 + Mfma<T>::row_of(v, lane), c = b * 16 + l15;
          if (full_mn || (m0 + wm0 + r < M && n0 + wn0 + c < N)) Cw2[(int64_t)r * P.ldc2 + c] = acc[a][b][v];
        }
  }
}

}  // namespace dla
