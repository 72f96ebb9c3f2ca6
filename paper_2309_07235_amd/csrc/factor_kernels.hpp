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

// Value of lane K of the caller's 16-lane row, for every lane of that row.
template <int K>
__device__ inline double row_bcast(double x) {
  int lo = __double2loint(x), hi = __double2hiint(x);
  lo = __builtin_amdgcn_update_dpp(0, lo, 0x150 + K, 0xF, 0xF, false);
  hi = __builtin_amdgcn_update_dpp(0, hi, 0x150 + K, 0xF, 0xF, false);
  return __hiloint2double(hi, lo);
}
template <int K>
__device__ inline float row_bcast(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x150 + K, 0xF, 0xF, false));
}

__device__ inline double fma_t(double a, double b, double c) { return __builtin_fma(a, b, c); }
__device__ inline float fma_t(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ inline double sqrt_t(double a) { return __builtin_sqrt(a); }
__device__ inline float sqrt_t(float a) { return __builtin_sqrtf(a); }

// ---- 16 x 16 register-level factorisations: lane i of a 16-lane row owns matrix row i ----

// In-place LU without pivoting of the block whose row i is a[0..15].  On exit
// a holds L (strict lower, unit diagonal implied) and U; rdiag[k] = 1/U[k][k]
// (same value in every lane).  zero_at: first k with an exactly zero pivot, or -1.
template <typename T>
__device__ inline void lu16(T (&a)[16], T (&rdiag)[16], int i, int& zero_at) {
  zero_at = -1;
  static_for<0, 16>([&](auto kc) {
    constexpr int k = decltype(kc)::value;
    const T piv = row_bcast<k>(a[k]);
    if (piv == T(0) && zero_at < 0) zero_at = k;
    const T rp = T(1) / piv;
    rdiag[k] = rp;
    const bool below = i > k;
    const T l = a[k] * rp;
    a[k] = below ? l : a[k];
    static_for<k + 1, 16>([&](auto jc) {
      constexpr int j = decltype(jc)::value;
      const T u = row_bcast<k>(a[j]);
      a[j] = below ? fma_t(-l, u, a[j]) : a[j];
    });
  });
}

// In-place Cholesky of the block whose lower-triangle row i is a[0..i].
// rdiag[k] = 1/L[k][k]; bad_at: first k whose pivot is not > 0, or -1.
template <typename T>
__device__ inline void chol16(T (&a)[16], T (&rdiag)[16], int i, int& bad_at) {
  bad_at = -1;
  static_for<0, 16>([&](auto kc) {
    constexpr int k = decltype(kc)::value;
    const T d = row_bcast<k>(a[k]);
    if (!(d > T(0)) && bad_at < 0) bad_at = k;
    const T s = sqrt_t(d);
    const T rs = T(1) / s;
    rdiag[k] = rs;
    const T l = (i == k) ? s : a[k] * rs;
    a[k] = (i >= k) ? l : a[k];
    static_for<k + 1, 16>([&](auto jc) {
      constexpr int j = decltype(jc)::value;
      const T ljk = row_bcast<j>(a[k]);  // L[j][k] lives in lane j
      a[j] = (i >= j) ? fma_t(-a[k], ljk, a[j]) : a[j];
    });
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
      const bool is = (i == k);
      static_for<0, k + 1>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        x[j] = is ? x[j] * rdiag[k] : x[j];
      });
    }
    const bool below = i > k;
    static_for<0, k + 1>([&](auto jc) {
      constexpr int j = decltype(jc)::value;
      const T v = row_bcast<k>(x[j]);
      x[j] = below ? fma_t(-a[k], v, x[j]) : x[j];
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
    const bool is = (i == k);
    static_for<k, 16>([&](auto jc) {
      constexpr int j = decltype(jc)::value;
      x[j] = is ? x[j] * rdiag[k] : x[j];
    });
    const bool above = i < k;
    static_for<k, 16>([&](auto jc) {
      constexpr int j = decltype(jc)::value;
      const T v = row_bcast<k>(x[j]);
      x[j] = above ? fma_t(-a[k], v, x[j]) : x[j];
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
  T* const S = reinterpret_cast<T*>(smem_raw);  // [kNbMax][kSld]
  T* const sRd = S + kNbMax * kSld;             // [kNbMax] reciprocals of the pivots
  __shared__ int s_info;

  const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l15 = lane & 15, l4 = lane >> 4;
  const int b = g.b;
  const int nblk = (b + kIb - 1) / kIb;
  const int bp = nblk * kIb;  // padded size: rows/columns b..bp-1 are identity

  if (tid == 0) s_info = 0;
  // ---- load, padding with the identity -------------------------------------------------
  for (int e = tid; e < bp * bp; e += kDiagThreads) {
    const int r = e / bp, c = e % bp;
    T v = (r == c) ? T(1) : T(0);
    if (r < b && c < b) v = g.A[(int64_t)r * g.lda + c];
    S[r * kSld + c] = v;
  }
  __syncthreads();

  for (int r = 0; r < nblk; ++r) {
    const int o = r * kIb;
    // ---- (a) 16 x 16 diagonal sub-block, wave 0 -----------------------------------------
    if (wave == 0) {
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
    }
    __syncthreads();
    const int rem = bp - o - kIb;  // rows/columns to the right of / below this sub-block
    if (rem > 0) {
      // ---- (b) inner panels: one thread per column (row panel) or per row (column panel) ----
      if (KIND == KIND_LU && tid < rem) {
        const int col = o + kIb + tid;
        T x[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = S[(o + i) * kSld + col];
#pragma unroll
        for (int k = 0; k < 15; ++k)
#pragma unroll
          for (int i = k + 1; i < 16; ++i) x[i] = fma_t(-S[(o + i) * kSld + o + k], x[k], x[i]);
#pragma unroll
        for (int i = 0; i < 16; ++i) S[(o + i) * kSld + col] = x[i];
      } else if (tid >= 256 && tid - 256 < rem) {
        const int row = o + kIb + (tid - 256);
        T x[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) x[j] = S[row * kSld + o + j];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          x[j] *= sRd[o + j];
#pragma unroll
          for (int jj = j + 1; jj < 16; ++jj) {
            // LU: U[j][jj];  Cholesky: (L^T)[j][jj] = L[jj][j]
            const T u = (KIND == KIND_LU) ? S[(o + j) * kSld + o + jj] : S[(o + jj) * kSld + o + j];
            x[jj] = fma_t(-x[j], u, x[jj]);
          }
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) S[row * kSld + o + j] = x[j];
      }
      __syncthreads();
      // ---- (c) inner trailing update on MFMA ------------------------------------------------
      const int nrem = rem / kIb;
      const int nwaves = kDiagThreads / 64;
      for (int q = wave; q < nrem * nrem; q += nwaves) {
        const int ci = q / nrem, di = q % nrem;
        if (KIND == KIND_CHOL && di > ci) continue;
        const int c0 = o + kIb + ci * kIb, d0 = o + kIb + di * kIb;
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
      }
      __syncthreads();
    }
  }

  // ---- inverses of the diagonal sub-blocks: one 16-lane row per sub-block -----------------
  // waves 0..1: lower factor, sub-blocks 4*wave + l4;  waves 2..3: upper factor (LU only)
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
  }

  // ---- store the factored block ------------------------------------------------------------
  for (int e = tid; e < b * b; e += kDiagThreads) {
    const int r = e / b, c = e % b;
    if (KIND == KIND_LU || c <= r) g.A[(int64_t)r * g.lda + c] = S[r * kSld + c];
  }
  if (tid == 0 && g.info) {
    if (g.k0 == 0) *g.info = s_info;            // first block of the call: initialise
    else if (s_info != 0 && *g.info == 0) *g.info = s_info;
  }
}

template <typename T>
constexpr int diag_lds_bytes() {
  return (kNbMax * kSld + kNbMax) * (int)sizeof(T);
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
  // tri_index(col block, row block)).  RIGHT/Cholesky needs L again.
  const bool want_upper = (!left) && KIND == KIND_LU;
  for (int t = 0; t < nblk * (nblk + 1) / 2; ++t) {
    int hi = 0;
    while ((hi + 1) * (hi + 2) / 2 <= t) ++hi;
    const int lo = t - hi * (hi + 1) / 2;
    const int rr = tid >> 4, cc = tid & 15;  // 256 threads = one element each
    T v;
    if (hi == lo) {
      v = (want_upper ? g.inv_up : g.inv_lo)[hi * 256 + rr * 16 + cc];
    } else {
      const int gr = (want_upper ? lo : hi) * kIb + rr, gc = (want_upper ? hi : lo) * kIb + cc;
      v = (gr < b && gc < b) ? -g.D[(int64_t)gr * g.lda + gc] : T(0);
    }
    Tri[t * kBlk + rr * (kIb + 1) + cc] = v;
  }
  __syncthreads();

  const int slice = ((left ? (int)blockIdx.x : (int)blockIdx.x - g.n_left) * (kTrsmThreads / 64) + wave) * kIb;
  if (slice >= m) return;

  acc_t acc[NB];
  if (left) {
    // ---------------- X = L11^-1 P : wave owns columns slice .. slice+15 ----------------
    T* const P = g.left + slice;
    const bool col_ok = slice + l15 < m;
#pragma unroll
    for (int s = 0; s < NB; ++s)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = s * kIb + Mfma<T>::row_of(v, lane);
        acc[s][v] = (s < nblk && row < b && col_ok) ? P[(int64_t)row * g.lda + l15] : T(0);
      }
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
#pragma unroll
    for (int s = 0; s < NB; ++s)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = s * kIb + Mfma<T>::row_of(v, lane);
        if (s < nblk && row < b && col_ok) P[(int64_t)row * g.lda + l15] = acc[s][v];
      }
  } else {
    // ---------------- X = P R^-1 : wave owns rows slice .. slice+15 ----------------
    T* const P = g.right + (int64_t)slice * g.lda;
#pragma unroll
    for (int c = 0; c < NB; ++c)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = Mfma<T>::row_of(v, lane), col = c * kIb + l15;
        acc[c][v] = (c < nblk && slice + row < m && col < b) ? P[(int64_t)row * g.lda + col] : T(0);
      }
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
#pragma unroll
    for (int c = 0; c < NB; ++c)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = Mfma<T>::row_of(v, lane), col = c * kIb + l15;
        if (c < nblk && slice + row < m && col < b) P[(int64_t)row * g.lda + col] = acc[c][v];
      }
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
