// Panel-phase kernels of the blocked right-looking factorisations (paper,
// Section "Linear Algebra Benchmarks": A = L*U without pivoting, A = L*L^T):
//
//   diag_kernel   one workgroup factors the b x b diagonal block (b <= 128) held
//                 in LDS, recursively in 16 x 16 sub-blocks: a wavefront-level
//                 16 x 16 factorisation in registers (one matrix row per lane,
//                 pivot row broadcast with DPP row_newbcast), register-level
//                 triangular solves for the 16-wide inner panels, MFMA for the
//                 inner trailing update.  It also inverts every 16 x 16
//                 diagonal sub-block; the inverses go to the workspace.
// The panel solves and the look-ahead head update, which consume those inverses,
// live in head_kernel.hpp.
#pragma once
#include <type_traits>
#include "dla_common.hpp"

namespace dla {

constexpr int kNbMax = 128;            // largest block size
constexpr int kIb = 16;                // inner block = one MFMA block
constexpr int kSld = kNbMax + 1;       // odd LDS row stride of the diagonal block
constexpr int kDiagThreads = 512;
constexpr int kBlk = kIb * (kIb + 1);  // 16 x 17: one padded 16 x 16 sub-block in LDS

enum FactorKind { KIND_LU = 0, KIND_CHOL = 1 };

template <int I, int N, typename F>
__device__ inline void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// Value of lane K of the caller's 16-lane row, for every lane of that row (DPP row_newbcast).
template <int K>
__device__ inline double row_bcast(double x) {
  return __builtin_amdgcn_update_dpp(x, x, 0x150 + K, 0xF, 0xF, true);  // every lane is written: no 'old' value needed
}
template <int K>
__device__ inline float row_bcast(float x) {
  return __builtin_amdgcn_update_dpp(x, x, 0x150 + K, 0xF, 0xF, true);
}

// acc -= (value of src in lane K of the caller's 16-lane row) * m, as one DPP multiply-add: the
// negation is a source modifier of the instruction, so it adds nothing to a dependent chain.
// The two wait states a DPP read needs after a VALU write of its source are part of the statement.
template <int K>
__device__ inline void fnmac_bcast(double& acc, double src, double m) {
  asm("s_nop 1\n\tv_fmac_f64_dpp %0, -%1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
      : "+v"(acc)
      : "v"(src), "v"(m), "n"(K));
}
template <int K>
__device__ inline void fnmac_bcast(float& acc, float src, float m) {
  asm("s_nop 1\n\tv_fmac_f32_dpp %0, -%1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
      : "+v"(acc)
      : "v"(src), "v"(m), "n"(K));
}

__device__ inline double fma_t(double a, double b, double c) { return __builtin_fma(a, b, c); }
__device__ inline float fma_t(float a, float b, float c) { return __builtin_fmaf(a, b, c); }

// Reciprocal and reciprocal square root from the hardware estimate plus Newton steps (about 1 ulp;
// exact for powers of two).  They sit on the dependent chain of every pivot, where an IEEE
// division or square root would cost twice as many dependent instructions.
__device__ inline double fast_rcp(double p) {
  double r = __builtin_amdgcn_rcp(p);
  double e = __builtin_fma(-p, r, 1.0);
  r = __builtin_fma(r, e, r);
  e = __builtin_fma(-p, r, 1.0);
  return __builtin_fma(r, e, r);
}
__device__ inline float fast_rcp(float p) {
  float r = __builtin_amdgcn_rcpf(p);
  const float e = __builtin_fmaf(-p, r, 1.0f);
  return __builtin_fmaf(r, e, r);
}
__device__ inline double rcp_estimate(double p) { return __builtin_amdgcn_rcp(p); }
__device__ inline float rcp_estimate(float p) { return __builtin_amdgcn_rcpf(p); }
template <typename T>
__device__ inline T rcp_refine(T p, T r) {  // one Newton step
  const T e = fma_t(-p, r, T(1));
  return fma_t(r, e, r);
}
__device__ inline double rsq_estimate(double d) { return __builtin_amdgcn_rsq(d); }
__device__ inline float rsq_estimate(float d) { return __builtin_amdgcn_rsqf(d); }
template <typename T>
__device__ inline T rsq_refine(T d, T y) {  // one Newton step towards 1/sqrt(d)
  const T t = fma_t(-d * y, y, T(1));
  return fma_t(T(0.5) * y, t, y);
}
// y ~ 1/sqrt(d) and s ~ sqrt(d)
__device__ inline void fast_rsqrt(double d, double& s, double& y) {
  y = __builtin_amdgcn_rsq(d);
  double t = __builtin_fma(-d * y, y, 1.0);
  y = __builtin_fma(0.5 * y, t, y);
  t = __builtin_fma(-d * y, y, 1.0);
  y = __builtin_fma(0.5 * y, t, y);
  s = d * y;
  s = __builtin_fma(__builtin_fma(-s, s, d), 0.5 * y, s);
}
__device__ inline void fast_rsqrt(float d, float& s, float& y) {
  y = __builtin_amdgcn_rsqf(d);
  const float t = __builtin_fmaf(-d * y, y, 1.0f);
  y = __builtin_fmaf(0.5f * y, t, y);
  s = d * y;
  s = __builtin_fmaf(__builtin_fmaf(-s, s, d), 0.5f * y, s);
}

__device__ inline double sqrt_t(double a) { return __builtin_sqrt(a); }
__device__ inline float sqrt_t(float a) { return __builtin_sqrtf(a); }

// ---- 16 x 16 register-level factorisations: lane i of a 16-lane row owns matrix row i ----

// In-place LU without pivoting of the block whose row i is a[0..15].  On exit
// a holds L (strict lower, unit diagonal implied) and U; rdiag[k] = 1/U[k][k]
// (same value in every lane).  zero_at: first k with an exactly zero pivot, or -1.
// Rows that do not take part in a step use a zero multiplier instead of a select.
template <typename T>
__device__ inline void lu16(T (&a)[16], T (&rdiag)[16], int i, int& zero_at) {
  zero_at = -1;
  T piv = row_bcast<0>(a[0]);
  T rp = fast_rcp(piv);
  static_for<0, 16>([&](auto kc) {
    constexpr int k = decltype(kc)::value;
    if (piv == T(0) && zero_at < 0) zero_at = k;
    rdiag[k] = rp;
    const bool below = i > k;
    const T l = below ? a[k] * rp : T(0);
    a[k] = below ? l : a[k];
    // Column k+1 first: it carries the next pivot, whose reciprocal (a chain of dependent
    // instructions) then overlaps with the independent updates of the remaining columns.
    if constexpr (k + 1 < 16) {
      fnmac_bcast<k>(a[k + 1], a[k + 1], l);
      piv = row_bcast<k + 1>(a[k + 1]);
      __builtin_amdgcn_sched_barrier(0);
      T r = rcp_estimate(piv);
      // interleave the Newton steps with the row updates, a few columns per step
      constexpr int rest = 14 - k;                 // columns k+2 .. 15
      constexpr int c1 = k + 2 + (rest + 3) / 4, c2 = k + 2 + (2 * rest + 3) / 4, c3 = k + 2 + (3 * rest + 3) / 4;
      static_for<k + 2, c1>([&](auto jc) { constexpr int j = decltype(jc)::value; fnmac_bcast<k>(a[j], a[j], l); });
      __builtin_amdgcn_sched_barrier(0);
      r = rcp_refine(piv, r);
      static_for<c1, c2>([&](auto jc) { constexpr int j = decltype(jc)::value; fnmac_bcast<k>(a[j], a[j], l); });
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (sizeof(T) == 8) r = rcp_refine(piv, r);
      static_for<c2, c3>([&](auto jc) { constexpr int j = decltype(jc)::value; fnmac_bcast<k>(a[j], a[j], l); });
      __builtin_amdgcn_sched_barrier(0);
      static_for<c3, 16>([&](auto jc) { constexpr int j = decltype(jc)::value; fnmac_bcast<k>(a[j], a[j], l); });
      rp = r;
    }
  });
}

// In-place Cholesky of the block whose lower-triangle row i is a[0..i]; a[j] for j > i is
// scratch (never read for a result, may hold anything).  rdiag[k] = 1/L[k][k];
// bad_at: first k whose pivot is not > 0, or -1.
template <typename T>
__device__ inline void chol16(T (&a)[16], T (&rdiag)[16], int i, int& bad_at) {
  bad_at = -1;
  T d = row_bcast<0>(a[0]);
  T s, rs;
  fast_rsqrt(d, s, rs);
  static_for<0, 16>([&](auto kc) {
    constexpr int k = decltype(kc)::value;
    if (!(d > T(0)) && bad_at < 0) bad_at = k;
    rdiag[k] = rs;
    const T l = (i == k) ? s : a[k] * rs;
    a[k] = (i >= k) ? l : a[k];
    // rows i <= k only touch their scratch entries a[j], j > k >= i, below.
    // Column k+1 first (next pivot), then its reciprocal square root interleaved with the rest.
    if constexpr (k + 1 < 16) {
      fnmac_bcast<k + 1>(a[k + 1], a[k], a[k]);  // a[j] -= L[i][k] * L[j][k]; L[j][k] lives in lane j
      d = row_bcast<k + 1>(a[k + 1]);
      __builtin_amdgcn_sched_barrier(0);
      T y = rsq_estimate(d);
      constexpr int rest = 14 - k;
      constexpr int c1 = k + 2 + (rest + 3) / 4, c2 = k + 2 + (2 * rest + 3) / 4, c3 = k + 2 + (3 * rest + 3) / 4;
      static_for<k + 2, c1>([&](auto jc) { constexpr int j = decltype(jc)::value; fnmac_bcast<j>(a[j], a[k], a[k]); });
      __builtin_amdgcn_sched_barrier(0);
      y = rsq_refine(d, y);
      static_for<c1, c2>([&](auto jc) { constexpr int j = decltype(jc)::value; fnmac_bcast<j>(a[j], a[k], a[k]); });
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (sizeof(T) == 8) y = rsq_refine(d, y);
      static_for<c2, c3>([&](auto jc) { constexpr int j = decltype(jc)::value; fnmac_bcast<j>(a[j], a[k], a[k]); });
      __builtin_amdgcn_sched_barrier(0);
      T sq = d * y;
      sq = fma_t(fma_t(-sq, sq, d), T(0.5) * y, sq);
      static_for<c3, 16>([&](auto jc) { constexpr int j = decltype(jc)::value; fnmac_bcast<j>(a[j], a[k], a[k]); });
      s = sq;
      rs = y;
    }
  });
}

// x = row i of the inverse of the lower-triangular matrix whose row i is a[0..i];
// UNIT: unit diagonal (a[i] ignored), else rdiag[k] = 1/diagonal.
template <typename T, bool UNIT>
__device__ inline void inv_lower16(const T (&a)[16], const T (&rdiag)[16], T (&x)[16], int i) {
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
      fnmac_bcast<k>(x[j], x[j], mult);
    });
  });
}

// x = row i of the inverse of the upper-triangular matrix whose row i is a[i..15].
template <typename T>
__device__ inline void inv_upper16(const T (&a)[16], const T (&rdiag)[16], T (&x)[16], int i) {
#pragma unroll
  for (int j = 0; j < 16; ++j) x[j] = (j == i) ? T(1) : T(0);
  static_for<0, 16>([&](auto kk) {
    constexpr int k = 15 - decltype(kk)::value;
    const T scale = (i == k) ? rdiag[k] : T(1);
    static_for<k, 16>([&](auto jc) {
      constexpr int j = decltype(jc)::value;
      x[j] *= scale;
    });
    const T mult = (i < k) ? a[k] : T(0);
    static_for<k, 16>([&](auto jc) {
      constexpr int j = decltype(jc)::value;
      fnmac_bcast<k>(x[j], x[j], mult);
    });
  });
}

// --------------------------------------------------------------------------------------
template <typename T>
struct DiagArgs {
  T* A;          // top-left element of the diagonal block
  int64_t lda;
  int b;         // actual block size (<= kNbMax)
  int k0;        // global index of the block's first row/column (for info)
  int* info;     // device, may be null
  T* inv_lo;     // out: nblk inverted 16 x 16 diagonal sub-blocks of L (row-major, 256 elements each)
  T* inv_up;     // out: same for U (LU only)
  // look-ahead pipeline only (null / 0 otherwise): the block is ready once *wait_counter >= wait_target
  // (head updates finished so far); on completion *done_counter is incremented
  const int* wait_counter;
  int wait_target;
  int* done_counter;
  int* broken;   // set by a wait that gave up (see chain_wait); reported as info = -1
  long long wait_ticks;  // how long a wait may last, in ticks of the constant-rate wall clock
};

template <typename T, int KIND>
__global__ void __launch_bounds__(kDiagThreads) diag_kernel(const DiagArgs<T> g) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  T* const S = reinterpret_cast<T*>(smem_raw);  // [kNbMax + 1][kSld]: row kNbMax and column kNbMax are dump space
  T* const sRd = S + (kNbMax + 1) * kSld;       // [kNbMax] reciprocals of the pivots
  __shared__ int s_info;
  constexpr int NWAVES = kDiagThreads / 64;

  const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l15 = lane & 15, l4 = lane >> 4;
  const int b = g.b;
  const int nblk = (b + kIb - 1) / kIb;
  const int bp = nblk * kIb;  // padded size: rows/columns b..bp-1 are identity

  if (g.wait_counter) chain_wait(g.wait_counter, g.wait_target, g.broken, g.wait_ticks, tid);
  if (tid == 0) s_info = 0;
  // ---- load, padding with the identity: thread = two adjacent columns, 8 rows per pass, all
  // loads issued before the first LDS store
  {
    constexpr int TPR = kNbMax / 2;             // threads per row
    constexpr int RPP = kDiagThreads / TPR;     // rows per pass
    constexpr int PASSES = kNbMax / RPP;
    const int c = (tid % TPR) * 2, r0 = tid / TPR;
    T v0[PASSES], v1[PASSES];
    // addresses are clamped into the block so every load is unconditional (no branch, no wait
    // between loads); out-of-block positions are replaced by the identity afterwards
    const int cc0 = c < b ? c : b - 1, cc1 = c + 1 < b ? c + 1 : b - 1;
#pragma unroll
    for (int it = 0; it < PASSES; ++it) {
      const int r = r0 + it * RPP;
      const T* p = g.A + (int64_t)(r < b ? r : b - 1) * g.lda;
      v0[it] = p[cc0];
      v1[it] = p[cc1];
    }
#pragma unroll
    for (int it = 0; it < PASSES; ++it) {
      const int r = r0 + it * RPP;
      if (!(r < b && c < b)) v0[it] = (r == c) ? T(1) : T(0);
      if (!(r < b && c + 1 < b)) v1[it] = (r == c + 1) ? T(1) : T(0);
    }
#pragma unroll
    for (int it = 0; it < PASSES; ++it) {
      const int r = r0 + it * RPP;
      if (r < bp && c < bp) {
        S[r * kSld + c] = v0[it];
        S[r * kSld + c + 1] = v1[it];
      }
    }
  }
  __syncthreads();

  // 16 x 16 diagonal sub-block at offset o: rows to registers, factor, back to LDS (one wave)
  auto factor_sub_block = [&](int o) {
    T a[16], rd[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) a[j] = S[(o + l15) * kSld + o + j];
    int bad;
    if (KIND == KIND_LU) lu16(a, rd, l15, bad);
    else chol16(a, rd, l15, bad);
    if (lane < 16) {
#pragma unroll
      for (int j = 0; j < 16; ++j)
        if (KIND == KIND_LU || j <= l15) S[(o + l15) * kSld + o + j] = a[j];
    }
    if (lane == 0) {
#pragma unroll
      for (int j = 0; j < 16; ++j) sRd[o + j] = rd[j];
      if (bad >= 0 && o + bad < b && s_info == 0) s_info = g.k0 + o + bad + 1;
    }
  };
  // one 16 x 16 block of the inner trailing update of the stage at offset o
  auto update_block = [&](int o, int c0, int d0) {
    typename Mfma<T>::acc_t acc;
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[v] = S[(c0 + Mfma<T>::row_of(v, lane)) * kSld + d0 + l15];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const T fa = -S[(c0 + l15) * kSld + o + kk * 4 + l4];
      const T fb = (KIND == KIND_LU) ? S[(o + kk * 4 + l4) * kSld + d0 + l15]
                                     : S[(d0 + l15) * kSld + o + kk * 4 + l4];
      acc = Mfma<T>::mma(fa, fb, acc);
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) S[(c0 + Mfma<T>::row_of(v, lane)) * kSld + d0 + l15] = acc[v];
  };

  // two independent blocks at once
  auto update_block2 = [&](int o, int c0, int d0, int c1, int d1) {
    typename Mfma<T>::acc_t acc0, acc1;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      acc0[v] = S[(c0 + Mfma<T>::row_of(v, lane)) * kSld + d0 + l15];
      acc1[v] = S[(c1 + Mfma<T>::row_of(v, lane)) * kSld + d1 + l15];
    }
    T fa0[4], fb0[4], fa1[4], fb1[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      fa0[kk] = -S[(c0 + l15) * kSld + o + kk * 4 + l4];
      fa1[kk] = -S[(c1 + l15) * kSld + o + kk * 4 + l4];
      fb0[kk] = (KIND == KIND_LU) ? S[(o + kk * 4 + l4) * kSld + d0 + l15] : S[(d0 + l15) * kSld + o + kk * 4 + l4];
      fb1[kk] = (KIND == KIND_LU) ? S[(o + kk * 4 + l4) * kSld + d1 + l15] : S[(d1 + l15) * kSld + o + kk * 4 + l4];
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      acc0 = Mfma<T>::mma(fa0[kk], fb0[kk], acc0);
      acc1 = Mfma<T>::mma(fa1[kk], fb1[kk], acc1);
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      S[(c0 + Mfma<T>::row_of(v, lane)) * kSld + d0 + l15] = acc0[v];
      S[(c1 + Mfma<T>::row_of(v, lane)) * kSld + d1 + l15] = acc1[v];
    }
  };

  if (wave == 0) factor_sub_block(0);
  __syncthreads();

  for (int r = 0; r + 1 < nblk; ++r) {
    const int o = r * kIb;
    const int rem = bp - o - kIb;  // rows/columns to the right of / below this sub-block
    // ---- inner panels: one thread per column (row panel) or per row (column panel).  The 16 x 16
    // factor is uniform over the panel, so each 16-lane row keeps it in registers (lane i = its
    // row i) and feeds the substitution through DPP broadcasts instead of LDS reads.
    if (KIND == KIND_LU && tid < 128) {
      // threads past the padded block work on the dump column, so the arithmetic stays unconditional
      const int col = tid < rem ? o + kIb + tid : kNbMax;
      T f[16], x[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) f[j] = S[(o + l15) * kSld + o + j];  // row l15 of L_rr \ U_rr
#pragma unroll
      for (int i = 0; i < 16; ++i) x[i] = S[(o + i) * kSld + col];
      static_for<0, 15>([&](auto kc) {
        constexpr int k = decltype(kc)::value;
        static_for<k + 1, 16>([&](auto ic) {
          constexpr int i = decltype(ic)::value;
          fnmac_bcast<i>(x[i], f[k], x[k]);  // x[i] -= L[i][k] * x[k]; L[i][k] = entry k of lane i
        });
        __builtin_amdgcn_sched_barrier(0);  // keep the broadcasts of later steps from being hoisted (registers)
      });
#pragma unroll
      for (int i = 0; i < 16; ++i) S[(o + i) * kSld + col] = x[i];
    } else if (tid >= 128 && tid < 256) {  // waves 2, 3: not the SIMDs of the row panel's waves 0, 1
      const int t = tid - 128;
      const int row = t < rem ? o + kIb + t : kNbMax;  // dump row for the idle threads
      T f[16], x[16], rd[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        f[j] = S[(o + l15) * kSld + o + j];
        rd[j] = sRd[o + j];
      }
#pragma unroll
      for (int j = 0; j < 16; ++j) x[j] = S[row * kSld + o + j];
      static_for<0, 16>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        x[j] *= rd[j];
        static_for<j + 1, 16>([&](auto qc) {
          constexpr int jj = decltype(qc)::value;
          // LU: U[j][jj] = entry jj of lane j;  Cholesky: (L^T)[j][jj] = L[jj][j] = entry j of lane jj
          if constexpr (KIND == KIND_LU) fnmac_bcast<j>(x[jj], f[jj], x[j]);
          else fnmac_bcast<jj>(x[jj], f[j], x[j]);
        });
        __builtin_amdgcn_sched_barrier(0);
      });
#pragma unroll
      for (int j = 0; j < 16; ++j) S[row * kSld + o + j] = x[j];
    }
    __syncthreads();
    // ---- inner trailing update on MFMA.  Wave 0 updates the next diagonal sub-block first and
    // factors it while the other waves update the remaining blocks (look-ahead inside the block).
    const int nrem = rem / kIb;
    if (wave == 0) {
      update_block(o, o + kIb, o + kIb);
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");  // this wave's LDS writes before its reads below
      factor_sub_block(o + kIb);
    } else {
      // q = 0 is wave 0's block; two blocks per iteration give the MFMA chains some overlap
      for (int q = wave; q < nrem * nrem; q += 2 * (NWAVES - 1)) {
        const int q2 = q + (NWAVES - 1);
        const int ci = q / nrem, di = q % nrem, ci2 = q2 / nrem, di2 = q2 % nrem;
        const bool do1 = !(KIND == KIND_CHOL && di > ci);
        const bool do2 = q2 < nrem * nrem && !(KIND == KIND_CHOL && di2 > ci2);
        if (do1 && do2) update_block2(o, o + kIb + ci * kIb, o + kIb + di * kIb, o + kIb + ci2 * kIb, o + kIb + di2 * kIb);
        else if (do1) update_block(o, o + kIb + ci * kIb, o + kIb + di * kIb);
        else if (do2) update_block(o, o + kIb + ci2 * kIb, o + kIb + di2 * kIb);
      }
    }
    __syncthreads();
  }

  // ---- inverses of the diagonal sub-blocks: one 16-lane row per sub-block ---------------------
  // waves 0..1: lower factor, sub-blocks 4*(wave&1) + l4;  waves 2..3: upper factor (LU only);
  // the other waves store the factored block meanwhile.
  if (wave < 4) {
    const bool lower = wave < 2;
    const int blk = (wave & 1) * 4 + l4;
    if (blk < nblk && (lower || KIND == KIND_LU)) {
      const int o = blk * kIb;
      T a[16], rd[16], x[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        a[j] = S[(o + l15) * kSld + o + j];
        rd[j] = sRd[o + j];
      }
      if (lower) inv_lower16<T, KIND == KIND_LU>(a, rd, x, l15);
      else inv_upper16<T>(a, rd, x, l15);
      T* out = (lower ? g.inv_lo : g.inv_up) + blk * 256 + l15 * 16;
#pragma unroll
      for (int j = 0; j < 16; ++j) out[j] = x[j];
    }
  } else {
    // 4 waves = 256 threads: thread = two adjacent columns, 4 rows per pass
    const int t = tid - 256;
    const int c = (t % (kNbMax / 2)) * 2, r0 = t / (kNbMax / 2);
    for (int r = r0; r < b; r += 4) {  // Cholesky: zeros above the diagonal (the output convention)
      T* p = g.A + (int64_t)r * g.lda + c;
      if (c < b) p[0] = (KIND == KIND_LU || c <= r) ? S[r * kSld + c] : T(0);
      if (c + 1 < b) p[1] = (KIND == KIND_LU || c + 1 <= r) ? S[r * kSld + c + 1] : T(0);
    }
  }
  if (tid == 0 && g.info) {
    if (g.k0 == 0) *g.info = s_info;  // first block of the call: initialise
    else if (s_info != 0 && *g.info == 0) *g.info = s_info;
    if (g.broken && __hip_atomic_load(g.broken, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) *g.info = -1;
  }
  if (g.done_counter) chain_signal(g.done_counter, 1, tid);
}

template <typename T>
constexpr int diag_lds_bytes() {
  return ((kNbMax + 1) * kSld + kNbMax) * (int)sizeof(T);
}

// Zero a few ints (the hand-over counters) with a kernel: usable under stream capture, unlike a memset node.
static __global__ void zero_ints_kernel(int* p, int n) {
  if ((int)threadIdx.x < n) p[threadIdx.x] = 0;
}

// One wave that waits in place until a hand-over counter reaches its target (bounded like every such wait): put in
// front of a kernel on a stream that would otherwise wait for another stream's event.
static __global__ void gate_kernel(const int* counter, int target, int* broken, long long wait_ticks) {
  chain_wait(counter, target, broken, wait_ticks, (int)threadIdx.x);
}

// A 16 x 16 identity and three zeroed counters (the hand-over self-test's input).
static __global__ void identity16_kernel(double* a, int* counters) {
  const int t = (int)threadIdx.x;
  a[t] = (t / 16 == t % 16) ? 1.0 : 0.0;
  if (t < 3) counters[t] = 0;
}

// Zero the strict upper triangle (Cholesky output convention).  nb = 1: all of it.  nb > 1: only the
// blocks above the block diagonal of width nb, which no kernel of the factorisation touches, so that
// this can run beside the first steps; the diagonal-block kernel zeroes its own block's upper part.
template <typename T>
__global__ void __launch_bounds__(256) zero_upper_kernel(T* A, int64_t lda, int n, int nb) {
  const int col = (int)blockIdx.x * 256 + (int)threadIdx.x;
  for (int row = (int)blockIdx.y; row < n; row += (int)gridDim.y)
    if (col >= (row / nb + 1) * nb && col < n) A[(int64_t)row * lda + col] = T(0);
}

}  // namespace dla
