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
//   trsm_kernel   the large panel solves U12 = L11^-1 A12, L21 = A21 U11^-1 and
//                 L21 = A21 L11^-T as blocked substitution on MFMA: each
//                 wavefront owns a 16-wide slice of the panel in accumulator
//                 registers, multiplies by the inverted diagonal sub-blocks and
//                 eliminates with the off-diagonal sub-blocks staged in LDS.
#pragma once
#include <type_traits>
#include "dla_common.hpp"

// Optional phase tracing for development harnesses; expands to nothing in the library build.
#ifndef DLA_TRACE
#define DLA_TRACE(i)
#endif

namespace dla {

constexpr int kNbMax = 128;            // largest block size
constexpr int kIb = 16;                // inner block = one MFMA block
constexpr int kSld = kNbMax + 1;       // odd LDS row stride of the diagonal block
constexpr int kDiagThreads = 512;
constexpr int kTrsmThreads = 256;
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

// acc += (value of src in lane K of the caller's 16-lane row) * m, as one DPP multiply-add.
// The two wait states a DPP read needs after a VALU write of its source are part of the statement.
template <int K>
__device__ inline void fmac_bcast(double& acc, double src, double m) {
  asm("s_nop 1\n\tv_fmac_f64_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
      : "+v"(acc)
      : "v"(src), "v"(m), "n"(K));
}
template <int K>
__device__ inline void fmac_bcast(float& acc, float src, float m) {
  asm("s_nop 1\n\tv_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
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
    const T nl = -l;
    a[k] = below ? l : a[k];
    // Column k+1 first: it carries the next pivot, whose reciprocal (a chain of dependent
    // instructions) then overlaps with the independent updates of the remaining columns.
    if constexpr (k + 1 < 16) {
      fmac_bcast<k>(a[k + 1], a[k + 1], nl);
      piv = row_bcast<k + 1>(a[k + 1]);
      __builtin_amdgcn_sched_barrier(0);
      T r = rcp_estimate(piv);
      // interleave the Newton steps with the row updates, a few columns per step
      constexpr int rest = 14 - k;                 // columns k+2 .. 15
      constexpr int c1 = k + 2 + (rest + 3) / 4, c2 = k + 2 + (2 * rest + 3) / 4, c3 = k + 2 + (3 * rest + 3) / 4;
      static_for<k + 2, c1>([&](auto jc) { constexpr int j = decltype(jc)::value; fmac_bcast<k>(a[j], a[j], nl); });
      __builtin_amdgcn_sched_barrier(0);
      r = rcp_refine(piv, r);
      static_for<c1, c2>([&](auto jc) { constexpr int j = decltype(jc)::value; fmac_bcast<k>(a[j], a[j], nl); });
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (sizeof(T) == 8) r = rcp_refine(piv, r);
      static_for<c2, c3>([&](auto jc) { constexpr int j = decltype(jc)::value; fmac_bcast<k>(a[j], a[j], nl); });
      __builtin_amdgcn_sched_barrier(0);
      static_for<c3, 16>([&](auto jc) { constexpr int j = decltype(jc)::value; fmac_bcast<k>(a[j], a[j], nl); });
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
    const T nak = -a[k];
    // rows i <= k only touch their scratch entries a[j], j > k >= i, below.
    // Column k+1 first (next pivot), then its reciprocal square root interleaved with the rest.
    if constexpr (k + 1 < 16) {
      fmac_bcast<k + 1>(a[k + 1], a[k], nak);  // a[j] -= L[i][k] * L[j][k]; L[j][k] lives in lane j
      d = row_bcast<k + 1>(a[k + 1]);
      __builtin_amdgcn_sched_barrier(0);
      T y = rsq_estimate(d);
      constexpr int rest = 14 - k;
      constexpr int c1 = k + 2 + (rest + 3) / 4, c2 = k + 2 + (2 * rest + 3) / 4, c3 = k + 2 + (3 * rest + 3) / 4;
      static_for<k + 2, c1>([&](auto jc) { constexpr int j = decltype(jc)::value; fmac_bcast<j>(a[j], a[k], nak); });
      __builtin_amdgcn_sched_barrier(0);
      y = rsq_refine(d, y);
      static_for<c1, c2>([&](auto jc) { constexpr int j = decltype(jc)::value; fmac_bcast<j>(a[j], a[k], nak); });
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (sizeof(T) == 8) y = rsq_refine(d, y);
      static_for<c2, c3>([&](auto jc) { constexpr int j = decltype(jc)::value; fmac_bcast<j>(a[j], a[k], nak); });
      __builtin_amdgcn_sched_barrier(0);
      T sq = d * y;
      sq = fma_t(fma_t(-sq, sq, d), T(0.5) * y, sq);
      static_for<c3, 16>([&](auto jc) { constexpr int j = decltype(jc)::value; fmac_bcast<j>(a[j], a[k], nak); });
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
    const T nmult = (i > k) ? -a[k] : T(0);
    static_for<0, k + 1>([&](auto jc) {
      constexpr int j = decltype(jc)::value;
      fmac_bcast<k>(x[j], x[j], nmult);
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
    const T nmult = (i < k) ? -a[k] : T(0);
    static_for<k, 16>([&](auto jc) {
      constexpr int j = decltype(jc)::value;
      fmac_bcast<k>(x[j], x[j], nmult);
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

  DLA_TRACE(0);
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

  DLA_TRACE(1);
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
  DLA_TRACE(2);

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
        const T nxk = -x[k];
        static_for<k + 1, 16>([&](auto ic) {
          constexpr int i = decltype(ic)::value;
          fmac_bcast<i>(x[i], f[k], nxk);  // x[i] -= L[i][k] * x[k]; L[i][k] = entry k of lane i
        });
        __builtin_amdgcn_sched_barrier(0);  // keep the broadcasts of later steps from being hoisted (registers)
      });
#pragma unroll
      for (int i = 0; i < 16; ++i) S[(o + i) * kSld + col] = x[i];
    } else if (tid >= 256 && tid < 384) {
      const int t = tid - 256;
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
        const T nxj = -x[j];
        static_for<j + 1, 16>([&](auto qc) {
          constexpr int jj = decltype(qc)::value;
          // LU: U[j][jj] = entry jj of lane j;  Cholesky: (L^T)[j][jj] = L[jj][j] = entry j of lane jj
          if constexpr (KIND == KIND_LU) fmac_bcast<j>(x[jj], f[jj], nxj);
          else fmac_bcast<jj>(x[jj], f[j], nxj);
        });
        __builtin_amdgcn_sched_barrier(0);
      });
#pragma unroll
      for (int j = 0; j < 16; ++j) S[row * kSld + o + j] = x[j];
    }
    __syncthreads();
    DLA_TRACE(3 + 2 * r);
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
    DLA_TRACE(4 + 2 * r);
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
    for (int r = r0; r < b; r += 4) {
      T* p = g.A + (int64_t)r * g.lda + c;
      if (c < b && (KIND == KIND_LU || c <= r)) p[0] = S[r * kSld + c];
      if (c + 1 < b && (KIND == KIND_LU || c + 1 <= r)) p[1] = S[r * kSld + c + 1];
    }
  }
  DLA_TRACE(20);
  if (tid == 0 && g.info) {
    if (g.k0 == 0) *g.info = s_info;  // first block of the call: initialise
    else if (s_info != 0 && *g.info == 0) *g.info = s_info;
  }
}

template <typename T>
constexpr int diag_lds_bytes() {
  return ((kNbMax + 1) * kSld + kNbMax) * (int)sizeof(T);
}

// --------------------------------------------------------------------------------------
// Panel solves.  JOB_LEFT:  X = L11^-1 * P,  P = b x m  (LU row panel, 16 columns per wave)
//                JOB_RIGHT: X = P * R^-1,   P = m x b  (16 rows per wave), R = U11 (LU) or L11^T (Cholesky)
template <typename T>
struct TrsmArgs {
  const T* D;       // factored diagonal block (top-left element), leading dimension lda
  T* left;          // row panel  (b x m), may be null when n_left == 0
  T* right;         // column panel (m x b)
  int64_t lda;
  int b, m;
  int n_left;       // workgroups [0, n_left) do the row panel, the rest the column panel
  const T* inv_lo;  // inverted diagonal sub-blocks of the lower factor
  const T* inv_up;  // inverted diagonal sub-blocks of the upper factor (LU)
};

__device__ inline int tri_index(int hi, int lo) { return hi * (hi + 1) / 2 + lo; }

template <typename T>
constexpr int trsm_lds_bytes() {
  constexpr int nb = kNbMax / kIb;
  return (nb * (nb + 1) / 2 * kBlk + (kTrsmThreads / 64) * kBlk) * (int)sizeof(T);
}

template <typename T, int KIND>
__global__ void __launch_bounds__(kTrsmThreads) trsm_kernel(const TrsmArgs<T> g) {
  constexpr int NB = kNbMax / kIb;  // 8
  extern __shared__ __align__(16) unsigned char smem_raw[];
  T* const Tri = reinterpret_cast<T*>(smem_raw);         // compact lower-triangular set of padded sub-blocks
  T* const scratch_all = Tri + NB * (NB + 1) / 2 * kBlk;  // one padded sub-block per wave
  using acc_t = typename Mfma<T>::acc_t;

  const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l15 = lane & 15, l4 = lane >> 4;
  const int b = g.b, m = g.m;
  const int nblk = (b + kIb - 1) / kIb;
  const bool left = (int)blockIdx.x < g.n_left;
  T* const scratch = scratch_all + wave * kBlk;

  // ---- stage the triangular factor: off-diagonal sub-blocks negated, diagonal ones inverted ----
  // LEFT needs L (strict lower blocks).  RIGHT/LU needs U (strict upper blocks, stored at
  // tri_index(col block, row block)).  RIGHT/Cholesky needs L again.  One element per thread and
  // sub-block; every load is issued before the first LDS store.
  const bool want_upper = (!left) && KIND == KIND_LU;
  DLA_TRACE(0);
  {
    const int rr = tid >> 4, cc = tid & 15;
    T v[NB * (NB + 1) / 2];
#pragma unroll
    for (int hi = 0; hi < NB; ++hi)
#pragma unroll
      for (int lo = 0; lo <= hi; ++lo) {
        const int t = hi * (hi + 1) / 2 + lo;
        // unconditional loads from clamped addresses; masked afterwards
        const int hc = hi < nblk ? hi : nblk - 1, lc = lo < nblk ? lo : nblk - 1;
        if (hi == lo) {
          v[t] = (want_upper ? g.inv_up : g.inv_lo)[hc * 256 + rr * 16 + cc];
        } else {
          const int gr = (want_upper ? lc : hc) * kIb + rr, gc = (want_upper ? hc : lc) * kIb + cc;
          const T x = g.D[(int64_t)(gr < b ? gr : b - 1) * g.lda + (gc < b ? gc : b - 1)];
          v[t] = (gr < b && gc < b) ? -x : T(0);
        }
      }
#pragma unroll
    for (int hi = 0; hi < NB; ++hi)
#pragma unroll
      for (int lo = 0; lo <= hi; ++lo)
        if (hi < nblk) Tri[(hi * (hi + 1) / 2 + lo) * kBlk + rr * (kIb + 1) + cc] = v[hi * (hi + 1) / 2 + lo];
  }
  __syncthreads();
  DLA_TRACE(1);

  const int slice = ((left ? (int)blockIdx.x : (int)blockIdx.x - g.n_left) * (kTrsmThreads / 64) + wave) * kIb;
  if (slice >= m) return;

  acc_t acc[NB];
  if (left) {
    // ---------------- X = L11^-1 P : wave owns columns slice .. slice+15 ----------------
    T* const P = g.left + slice;
    const bool col_ok = slice + l15 < m;
    const int colc = col_ok ? l15 : m - 1 - slice;  // clamped: loads are unconditional, masked afterwards
#pragma unroll
    for (int s = 0; s < NB; ++s)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = s * kIb + Mfma<T>::row_of(v, lane);
        const T x = P[(int64_t)(row < b ? row : b - 1) * g.lda + colc];
        acc[s][v] = (row < b && col_ok) ? x : T(0);
      }
    DLA_TRACE(2);
#pragma unroll
    for (int r = 0; r < NB; ++r) {
      if (r < nblk) {
        // right-hand operand fragments of X_r: rows 4*kk + l4, column l15
        T fb[4];
        auto to_b = [&](const acc_t& x) {
          if constexpr (std::is_same<T, double>::value) {
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) fb[kk] = x[kk];  // fp64 result layout == B layout of k-step kk
          } else {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
#pragma unroll
            for (int v = 0; v < 4; ++v) scratch[Mfma<T>::row_of(v, lane) * (kIb + 1) + l15] = x[v];
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) fb[kk] = scratch[(kk * 4 + l4) * (kIb + 1) + l15];
          }
        };
        to_b(acc[r]);
        acc_t xr = {0, 0, 0, 0};
        const T* dblk = Tri + tri_index(r, r) * kBlk + l15 * (kIb + 1) + l4;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) xr = Mfma<T>::mma(dblk[kk * 4], fb[kk], xr);
        acc[r] = xr;
        to_b(xr);
#pragma unroll
        for (int s = r + 1; s < NB; ++s) {
          if (s < nblk) {
            const T* oblk = Tri + tri_index(s, r) * kBlk + l15 * (kIb + 1) + l4;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) acc[s] = Mfma<T>::mma(oblk[kk * 4], fb[kk], acc[s]);
          }
        }
      }
    }
    DLA_TRACE(3);
#pragma unroll
    for (int s = 0; s < NB; ++s)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = s * kIb + Mfma<T>::row_of(v, lane);
        if (s < nblk && row < b && col_ok) P[(int64_t)row * g.lda + l15] = acc[s][v];
      }
    DLA_TRACE(4);
  } else {
    // ---------------- X = P R^-1 : wave owns rows slice .. slice+15 ----------------
    T* const P = g.right + (int64_t)slice * g.lda;
#pragma unroll
    for (int c = 0; c < NB; ++c)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = Mfma<T>::row_of(v, lane), col = c * kIb + l15;
        const T x = P[(int64_t)(slice + row < m ? row : m - 1 - slice) * g.lda + (col < b ? col : b - 1)];
        acc[c][v] = (slice + row < m && col < b) ? x : T(0);
      }
    DLA_TRACE(5);
#pragma unroll
    for (int c = 0; c < NB; ++c) {
      if (c < nblk) {
        // left-hand operand fragments of a result block: rows l15, columns 4*kk + l4 (through LDS)
        T fa[4];
        auto to_a = [&](const acc_t& x) {
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
#pragma unroll
          for (int v = 0; v < 4; ++v) scratch[Mfma<T>::row_of(v, lane) * (kIb + 1) + l15] = x[v];
          __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) fa[kk] = scratch[l15 * (kIb + 1) + kk * 4 + l4];
        };
        // right-hand operand fragment of sub-block (row block s, column block d) of R, k-step kk
        auto rfrag = [&](int s, int d, int kk) -> T {
          const T* blk = Tri + tri_index(d, s) * kBlk;
          if (KIND == KIND_LU) return blk[(kk * 4 + l4) * (kIb + 1) + l15];  // U stored as is
          return blk[l15 * (kIb + 1) + kk * 4 + l4];                         // L stored; R = L^T
        };
        to_a(acc[c]);
        acc_t xc = {0, 0, 0, 0};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) xc = Mfma<T>::mma(fa[kk], rfrag(c, c, kk), xc);
        acc[c] = xc;
        to_a(xc);
#pragma unroll
        for (int d = c + 1; d < NB; ++d) {
          if (d < nblk) {
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) acc[d] = Mfma<T>::mma(fa[kk], rfrag(c, d, kk), acc[d]);
          }
        }
      }
    }
    DLA_TRACE(6);
#pragma unroll
    for (int c = 0; c < NB; ++c)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = Mfma<T>::row_of(v, lane), col = c * kIb + l15;
        if (c < nblk && slice + row < m && col < b) P[(int64_t)row * g.lda + col] = acc[c][v];
      }
    DLA_TRACE(7);
  }
}

// Zero the strict upper triangle (Cholesky output convention).
template <typename T>
__global__ void __launch_bounds__(256) zero_upper_kernel(T* A, int64_t lda, int n) {
  const int col = (int)blockIdx.x * 256 + (int)threadIdx.x;
  for (int row = (int)blockIdx.y; row < n; row += (int)gridDim.y)
    if (col > row && col < n) A[(int64_t)row * lda + col] = T(0);
}

}  // namespace dla
