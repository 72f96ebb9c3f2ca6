// Head update of the look-ahead pipeline.  After diagonal block k is factored, the only part of
// the trailing matrix the NEXT diagonal block waits for is
//     A[k+1][k+1] -= (A[k+1][k] * R^-1) * (L11^-1 * A[k][k+1])          (LU,  R = U11)
//     A[k+1][k+1] -= (A[k+1][k] * L11^-T) * (A[k+1][k] * L11^-T)^T      (Cholesky)
// This kernel computes exactly that b x b piece (a step of the blocked form of the decompositions
// A = L*U and A = L*L^T of the paper's Section "Linear Algebra Benchmarks"; the blocking is this
// library's, not the paper's) straight from the un-solved panel heads, so the
// next diagonal block can be factored while the full panel solves and the rest of the update run
// on other streams.  The panel heads are only read, and may be given as copies, so the panel solve
// that overwrites them in the matrix need not wait for this kernel.
//
// One workgroup of four wavefronts per 32 x 32 tile of the block.  The triangular factors (off-
// diagonal 16 x 16 sub-blocks as they are, diagonal ones inverted) are staged in LDS with ONE round
// of global loads, issued together with the right-hand sides and the tile itself, because this
// kernel runs beside a bulk update that keeps the memory system busy: every further round trip
// to global memory would cost microseconds on the latency chain.  Each wave then solves one
// triangular system for a 16-wide slice in accumulator registers, as blocked forward substitution
// on MFMA:
//   - both systems are written as  X = M^-1 * P  with M lower triangular (for  Y = P * R^-1  the
//     transposed system  Y^T = R^-T * P^T  is solved), so a result block is directly the
//     right-hand MFMA operand of the following products;
//   - the k index of every product is dealt to the lanes as k = 4 * (lane / 16) + kk for MFMA
//     step kk, so that the four values a lane feeds into the four steps are the four registers of
//     a result block.  For fp64 this needs the rows of the LEFT operand permuted (lane i supplies
//     logical row 4 * (i % 4) + i / 4), which costs nothing because those fragments are read
//     from LDS at arbitrary addresses anyway.
// In that layout the solved slices are also the operands of the final 16 x 16 x b products; they
// are exchanged between the waves through LDS (reusing the factor's space).
#pragma once
#include "factor_kernels.hpp"

namespace dla {

constexpr int kHeadThreads = 256;
constexpr int kHeadTile = 32;  // tile edge of one workgroup

template <typename T>
struct HeadArgs {
  const T* D;       // factored diagonal block k (b x b)
  const T* top;     // LU: block (k, k+1), b x bn.  Cholesky: unused
  const T* side;    // block (k+1, k), bn x b
  T* C;             // block (k+1, k+1), bn x bn
  int64_t lda;      // leading dimension of D and C
  int64_t ldh;      // leading dimension of top and side (they may be copies outside the matrix)
  int b, bn;        // b: multiple of 16, <= kNbMax;  1 <= bn <= kNbMax
  const T* inv_lo;  // inverted diagonal sub-blocks of the lower factor
  const T* inv_up;  // inverted diagonal sub-blocks of the upper factor (LU)
  // D and the inverses are ready once *wait_counter >= wait_target (diagonal blocks factored so far);
  // every workgroup increments *done_counter when its tile is stored
  // (both null when the streams order the two kernels instead)
  const int* wait_counter;
  int wait_target;
  int* done_counter;
  int* broken;      // set by a wait that gave up (see chain_wait)
  long long wait_ticks;  // how long the wait may last, in ticks of the constant-rate wall clock
};

template <typename T, int KIND>
constexpr int head_lds_bytes() {
  constexpr int nb = kNbMax / kIb;
  return (KIND == KIND_LU ? 2 : 1) * (nb * (nb + 1) / 2) * kBlk * (int)sizeof(T);
}

// lane (of the 16 that supply the rows of a left operand) -> logical row of the 16 x 16 block
template <typename T>
__device__ inline int head_prow(int l15) {
  if constexpr (sizeof(T) == 8) return ((l15 & 3) << 2) | (l15 >> 2);
  else return l15;
}

// X = M^-1 * P for a lower-triangular M whose sub-block (s, r), s >= r, sits at tri[s * (s + 1) / 2 + r]
// (diagonal ones inverted); element (i, k) of a sub-block at i * rs + k * cs.  acc holds P on entry
// and X on return: register v of acc[s] is row 16 * s + 4 * (lane / 16) + v, column lane % 16.
template <typename T, bool FULL>
__device__ inline void head_solve(const T* tri, int rs, int cs, int nblk, int lane,
                                  typename Mfma<T>::acc_t (&acc)[kNbMax / kIb]) {
  constexpr int NB = kNbMax / kIb;
  using acc_t = typename Mfma<T>::acc_t;
  const int l15 = lane & 15, l4 = lane >> 4;
  const T* const base = tri + head_prow<T>(l15) * rs + 4 * l4 * cs;
  static_for<0, NB>([&](auto rc) {
    constexpr int r = decltype(rc)::value;
    if (FULL || r < nblk) {
      const T* d = base + (r * (r + 1) / 2 + r) * kBlk;
      acc_t x = {0, 0, 0, 0};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) x = Mfma<T>::mma(d[kk * cs], acc[r][kk], x);
      acc[r] = x;
      T nx[4];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) nx[kk] = -x[kk];
      static_for<r + 1, NB>([&](auto sc) {
        constexpr int s = decltype(sc)::value;
        if (FULL || s < nblk) {
          const T* o = base + (s * (s + 1) / 2 + r) * kBlk;
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) acc[s] = Mfma<T>::mma(o[kk * cs], nx[kk], acc[s]);
        }
      });
    }
  });
}

template <typename T, int KIND>
__global__ void __launch_bounds__(kHeadThreads) head_kernel(const HeadArgs<T> g) {
  constexpr int NB = kNbMax / kIb;
  constexpr int NTRI = NB * (NB + 1) / 2;
  using acc_t = typename Mfma<T>::acc_t;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  T* const triL = reinterpret_cast<T*>(smem_raw);  // lower factor
  T* const triU = triL + NTRI * kBlk;              // upper factor (LU): sub-block (lo, hi) of U at slot hi * (hi + 1) / 2 + lo
  T* const slices = triL;                          // after the solves: 4 slices of NB * 4 * 64 values

  const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l15 = lane & 15, l4 = lane >> 4;
  const int b = g.b, bn = g.bn, nblk = b / kIb;
  const int64_t lda = g.lda;
  const int nt = (bn + kHeadTile - 1) / kHeadTile;
  int ti, tj;
  if (KIND == KIND_LU) {
    ti = (int)blockIdx.x / nt;
    tj = (int)blockIdx.x % nt;
  } else {  // lower-triangular tile set, row by row
    const int id = (int)blockIdx.x;
    int i = (int)((sqrtf(8.0f * (float)id + 1.0f) - 1.0f) * 0.5f);
    while (i * (i + 1) / 2 > id) --i;
    while ((i + 1) * (i + 2) / 2 <= id) ++i;
    ti = i;
    tj = id - i * (i + 1) / 2;
  }

  // ---- this wave's 16 x 16 piece of the tile, requested first ----------------------------------
  const int sub_r = ti * kHeadTile + (wave >> 1) * kIb, sub_c = tj * kHeadTile + (wave & 1) * kIb;
  const bool sub_on = sub_r < bn && sub_c < bn && !(KIND == KIND_CHOL && sub_c > sub_r);
  const int rows_valid = bn - sub_r < kIb ? bn - sub_r : kIb, cols_valid = bn - sub_c < kIb ? bn - sub_c : kIb;
  acc_t c = {0, 0, 0, 0};
  T* const Ct = g.C + (int64_t)sub_r * lda + sub_c;
  if (sub_on) {
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int r = Mfma<T>::row_of(v, lane);
      c[v] = Ct[(int64_t)(r < rows_valid ? r : rows_valid - 1) * lda + (l15 < cols_valid ? l15 : cols_valid - 1)];
    }
  }

  // ---- this wave's triangular system: right-hand side into the accumulators --------------------
  // LU:       waves 0, 1: X = L11^-1 * top[:, slice]          (slices of the tile's columns)
  //           waves 2, 3: Y^T = U11^-T * side[slice, :]^T     (slices of the tile's rows)
  // Cholesky: waves 0, 1: Y^T = L11^-1 * side[slice, :]^T for the tile's rows, waves 2, 3 for its columns
  const bool x_job = KIND == KIND_LU && wave < 2;
  const bool upper_job = KIND == KIND_LU && wave >= 2;
  int slice0;
  if (KIND == KIND_LU) slice0 = (wave < 2 ? tj : ti) * kHeadTile + (wave & 1) * kIb;
  else slice0 = (wave < 2 ? ti : tj) * kHeadTile + (wave & 1) * kIb;
  const bool job_on = slice0 < bn;
  acc_t acc[NB];
  {
    const int t_valid = bn - slice0 < kIb ? bn - slice0 : kIb;
    const int t = slice0 + (l15 < t_valid ? l15 : t_valid - 1);
    // element (k, t) of the right-hand side: top[k][t] for the X job, side[t][k] otherwise
    const T* const prhs = x_job ? g.top + (int64_t)(4 * l4) * g.ldh + t : g.side + (int64_t)t * g.ldh + 4 * l4;
    const int64_t ks = x_job ? g.ldh : 1;
#pragma unroll
    for (int s = 0; s < NB; ++s) {
      if (job_on && s < nblk) {
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[s][v] = prhs[(int64_t)(s * kIb + v) * ks];
      } else {
        acc[s] = acc_t{0, 0, 0, 0};
      }
    }
  }

  // The panel heads and the tile (requested above) do not depend on the diagonal block of this step,
  // the factors below do: the kernel is launched while that block is still being factored.
  if (g.wait_counter) chain_wait(g.wait_counter, g.wait_target, g.broken, g.wait_ticks, tid);

  // ---- stage the factors: one element per thread and sub-block, all loads before the first LDS store
  {
    const int rr = tid >> 4, cc = tid & 15;
    T vl[NTRI], vu[KIND == KIND_LU ? NTRI : 1];
#pragma unroll
    for (int hi = 0; hi < NB; ++hi)
#pragma unroll
      for (int lo = 0; lo <= hi; ++lo) {
        const int t = hi * (hi + 1) / 2 + lo;
        if (hi < nblk) {  // uniform
          if (hi == lo) {
            vl[t] = g.inv_lo[hi * 256 + rr * 16 + cc];
            if (KIND == KIND_LU) vu[t] = g.inv_up[hi * 256 + rr * 16 + cc];
          } else {
            vl[t] = g.D[(int64_t)(hi * kIb + rr) * lda + lo * kIb + cc];
            if (KIND == KIND_LU) vu[t] = g.D[(int64_t)(lo * kIb + rr) * lda + hi * kIb + cc];
          }
        }
      }
#pragma unroll
    for (int hi = 0; hi < NB; ++hi)
#pragma unroll
      for (int lo = 0; lo <= hi; ++lo) {
        const int t = hi * (hi + 1) / 2 + lo;
        if (hi < nblk) {
          triL[t * kBlk + rr * (kIb + 1) + cc] = vl[t];
          if (KIND == KIND_LU) triU[t * kBlk + rr * (kIb + 1) + cc] = vu[t];
        }
      }
  }
  __syncthreads();

  if (job_on) {
    // lower factor: element (i, k) of a sub-block at i * 17 + k; upper factor, transposed: at k * 17 + i
    const T* tri = upper_job ? triU : triL;
    const int rs = upper_job ? 1 : kIb + 1, cs = upper_job ? kIb + 1 : 1;
    if (nblk == NB) head_solve<T, true>(tri, rs, cs, nblk, lane, acc);
    else head_solve<T, false>(tri, rs, cs, nblk, lane, acc);
  }
  __syncthreads();  // every wave is done with the factors: their space takes the solved slices
#pragma unroll
  for (int s = 0; s < NB; ++s)
#pragma unroll
    for (int v = 0; v < 4; ++v) slices[(wave * NB * 4 + s * 4 + v) * 64 + lane] = acc[s][v];
  __syncthreads();
  if (sub_on) {
  // C piece -= Y * X over k = 0 .. b-1.  Left operand: lane (l4, i) holds Y[i][k]; right operand:
  // lane (l4, n) holds X[k][n]; k = 16 * s + 4 * l4 + v for step (s, v) in both.
  // LU: Y slices come from waves 2, 3 and X slices from waves 0, 1.  Cholesky: rows from 0, 1, columns from 2, 3.
  const int wy = (KIND == KIND_LU ? 2 : 0) + (wave >> 1), wx = (KIND == KIND_LU ? 0 : 2) + (wave & 1);
  const T* const sy = slices + (wy * NB * 4) * 64 + lane;
  const T* const sxp = slices + (wx * NB * 4) * 64 + lane;
#pragma unroll
  for (int s = 0; s < NB; ++s) {
    if (s < nblk) {
#pragma unroll
      for (int v = 0; v < 4; ++v) c = Mfma<T>::mma(-sy[(s * 4 + v) * 64], sxp[(s * 4 + v) * 64], c);
    }
  }
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int r = Mfma<T>::row_of(v, lane);
    if (r < rows_valid && l15 < cols_valid) Ct[(int64_t)r * lda + l15] = c[v];
  }
  }
  if (g.done_counter) chain_signal(g.done_counter, 1, tid);
}

// --------------------------------------------------------------------------------------
// Panel solves with the same machinery: U12 = L11^-1 * A12 (LU row panel, 16 columns per wave) and
// L21 = A21 * R^-1 (column panel, 16 rows per wave; R = U11 for LU, L11^T for Cholesky), the latter
// as the transposed system, so a lane reads and writes runs of four consecutive elements of its
// row and no result block has to be transposed through LDS.
constexpr int kSolveThreads = 256;

template <typename T>
struct SolveArgs {
  const T* D;       // factored diagonal block (b x b), leading dimension lda
  T* top;           // row panel  (b x m), LU only
  T* side;          // column panel (m x b)
  int64_t lda;
  int b, m;         // b: multiple of 16, <= kNbMax
  int n_top;        // workgroups [0, n_top) solve the row panel, the rest the column panel
  const T* inv_lo;
  const T* inv_up;
};

template <typename T>
constexpr int solve_lds_bytes() {
  constexpr int nb = kNbMax / kIb;
  return (nb * (nb + 1) / 2) * kBlk * (int)sizeof(T);
}

template <typename T, int KIND>
__global__ void __launch_bounds__(kSolveThreads) solve_kernel(const SolveArgs<T> g) {
  constexpr int NB = kNbMax / kIb;
  constexpr int NTRI = NB * (NB + 1) / 2;  // the 36 sub-blocks of the factor
  using acc_t = typename Mfma<T>::acc_t;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  T* const tri = reinterpret_cast<T*>(smem_raw);

  const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l15 = lane & 15, l4 = lane >> 4;
  const int b = g.b, m = g.m, nblk = b / kIb;
  const int64_t lda = g.lda;
  const bool x_job = KIND == KIND_LU && (int)blockIdx.x < g.n_top;
  const bool upper = KIND == KIND_LU && !x_job;  // the factor this workgroup needs: U (as U^T), else L
  const int wg = x_job ? (int)blockIdx.x : (int)blockIdx.x - g.n_top;
  const int slice0 = (wg * (kSolveThreads / 64) + wave) * kIb;
  const bool job_on = slice0 < m;

  // ---- right-hand side into the accumulators: element (k, t) is top[k][t] or side[t][k] ---------
  const int t_valid = m - slice0 < kIb ? m - slice0 : kIb;
  const int t = slice0 + (l15 < t_valid ? l15 : t_valid - 1);
  T* const prhs = x_job ? g.top + (int64_t)(4 * l4) * lda + t : g.side + (int64_t)t * lda + 4 * l4;
  const int64_t ks = x_job ? lda : 1;
  // A lane of the column panel's job owns runs of four consecutive elements of its row: read and written as
  // pairs where the panel's alignment allows (16 rows per instruction cost the texture path 16 look-ups
  // whatever the width, so half the instructions is half the look-ups).
  using vec2_t = typename Mfma<T>::vec2_t;
  const bool pairs = !x_job && lda % 2 == 0 && (uintptr_t)g.side % (2 * sizeof(T)) == 0;  // uniform
  acc_t acc[NB];
#pragma unroll
  for (int s = 0; s < NB; ++s) {
    if (job_on && s < nblk) {
      if (pairs) {
        const vec2_t lo = *reinterpret_cast<const vec2_t*>(prhs + s * kIb), hi = *reinterpret_cast<const vec2_t*>(prhs + s * kIb + 2);
        acc[s] = acc_t{lo[0], lo[1], hi[0], hi[1]};
      } else {
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[s][v] = prhs[(int64_t)(s * kIb + v) * ks];
      }
    } else {
      acc[s] = acc_t{0, 0, 0, 0};
    }
  }

  // ---- stage the factor: every load issued before the first LDS store (one round trip to memory; the
  // staging registers are free, LDS already holds the workgroups of a compute unit to two) ---------
  {
    const int rr = tid >> 4, cc = tid & 15;
    const T* const inv = upper ? g.inv_up : g.inv_lo;
    T v[NTRI];
#pragma unroll
    for (int hi = 0; hi < NB; ++hi)
#pragma unroll
      for (int lo = 0; lo <= hi; ++lo) {
        const int tb = hi * (hi + 1) / 2 + lo;
        if (hi < nblk) {  // uniform
          if (hi == lo) v[tb] = inv[hi * 256 + rr * 16 + cc];
          else if (upper) v[tb] = g.D[(int64_t)(lo * kIb + rr) * lda + hi * kIb + cc];
          else v[tb] = g.D[(int64_t)(hi * kIb + rr) * lda + lo * kIb + cc];
        }
      }
#pragma unroll
    for (int hi = 0; hi < NB; ++hi)
#pragma unroll
      for (int lo = 0; lo <= hi; ++lo) {
        const int tb = hi * (hi + 1) / 2 + lo;
        if (hi < nblk) tri[tb * kBlk + rr * (kIb + 1) + cc] = v[tb];
      }
  }
  __syncthreads();
  if (!job_on) return;
  {
    const int rs = upper ? 1 : kIb + 1, cs = upper ? kIb + 1 : 1;
    if (nblk == NB) head_solve<T, true>(tri, rs, cs, nblk, lane, acc);
    else head_solve<T, false>(tri, rs, cs, nblk, lane, acc);
  }
  if (l15 < t_valid) {
#pragma unroll
    for (int s = 0; s < NB; ++s) {
      if (s < nblk) {
        if (pairs) {
          *reinterpret_cast<vec2_t*>(prhs + s * kIb) = vec2_t{acc[s][0], acc[s][1]};
          *reinterpret_cast<vec2_t*>(prhs + s * kIb + 2) = vec2_t{acc[s][2], acc[s][3]};
        } else {
#pragma unroll
          for (int v = 0; v < 4; ++v) prhs[(int64_t)(s * kIb + v) * ks] = acc[s][v];
        }
      }
    }
  }
}

}  // namespace dla
