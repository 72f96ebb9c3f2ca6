// Skinny subtracting products for latency chains (the block steps of the solves with the factors;
// paper, Section "Introduction": LU and Cholesky are named as the factorisations behind solving
// systems of linear equations):  C (M x N) -= A (M x K) * B (K x N)  with few columns and K <= 512,
// where the launch is one link of a chain of dependent launches and what matters is how soon it ends.
//
// A 16 x 16 block of such a product is K / 4 dependent fp64 MFMAs, 64 cycles each: 3.4 us for K = 512
// on one SIMD, whatever the tile shape around it.  So a workgroup owns ONE 16 x 16 block and its four
// waves (one per SIMD) split the k range: every lane loads its whole share of both operands straight
// from global memory with all loads in flight at once (one round trip; no LDS staging, no slab loop),
// each wave multiplies a quarter of the k range, waves 1..3 leave their partial blocks in LDS and wave 0
// adds them in a fixed order, subtracts the sum from C and stores.  The result does not depend on
// the launch shape or on timing.
//
// k is dealt round-robin in pairs: with S = ceil(K / 16) steps per wave (rounded up to even), the lane group
// l4 (= lane / 16, the MFMA's k index) of wave w takes k = 32 t + 8 w + 2 l4 and the k after it for the steps
// 2 t and 2 t + 1.  A row-major left operand costs the texture path one look-up per row and load
// instruction, 16 per instruction where the right operand costs 4 (16 consecutive elements of 4 rows), and
// that path is what co-resident workgroups queue for; so a lane reads its pair of k with one load where
// the operand's alignment allows (base and leading dimension multiples of two elements).
//
// A launch carries up to kSkinnyMaxParts independent products (blocks of all of them in one grid).
// AT: the left operand is stored K x M (read transposed).
#pragma once
#include "dla_common.hpp"

namespace dla {

constexpr int kSkinnyMaxParts = 4;
constexpr int kSkinnyThreads = 256;
constexpr int kSkinnyMaxK = 512;

template <typename T>
struct SkinnyPart {
  const T* A;
  const T* B;
  T* C;
  T* C2;  // optional second destination of the result (leading dimension ldc2), or null
  int64_t lda, ldb, ldc, ldc2;
  int M, N, K;
  int tiles_n;     // workgroups per block row: 16-column blocks, or pairs of them (wide)
  int tile_begin;  // first workgroup of this product (skinny_workgroups() of them)
  int wide;        // 1: a workgroup owns two adjacent 16-column blocks (K <= 256 only)
};

// Workgroups of a product with M rows and tiles_n workgroups per block row (block rows padded to groups of kNumXcd).
inline int skinny_workgroups(int64_t M, int tiles_n) {
  const int tiles_m = (int)((M + 15) / 16);
  return (tiles_m + kNumXcd - 1) / kNumXcd * kNumXcd * tiles_n;
}

template <typename T>
struct SkinnyGroup {
  SkinnyPart<T> part[kSkinnyMaxParts];
  int nparts;
};

// The work of one workgroup: block `local` of product P, 16 rows x 16 NB columns.
// SMAX: steps per wave the code is built for (16 SMAX >= K).  NB: column blocks per workgroup; they share
// the left operand's loads, which pays where the left operand is the large one and the blocks are many.
template <typename T, bool AT, int SMAX, int NB>
__device__ __forceinline__ void skinny_block(const SkinnyPart<T>& P, const int local, T* __restrict__ red) {
  using acc_t = typename Mfma<T>::acc_t;
  // Workgroups are dealt to the XCDs round-robin; the column tiles of one block row are kXcdStride workgroups
  // apart so that they meet in one XCD's L2 (they read the same rows of the left operand).  A product's
  // workgroup count is padded to whole groups of kNumXcd block rows; the padding has nothing to do.
  const int ti = (local / (kNumXcd * P.tiles_n)) * kNumXcd + local % kNumXcd, tj = (local / kNumXcd) % P.tiles_n;
  if (ti * 16 >= P.M) return;  // uniform
  const int m0 = ti * 16, n0 = tj * (16 * NB);
  const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l15 = lane & 15, l4 = lane >> 4;
  const int M = P.M, N = P.N, K = P.K;
  const int S = (K + 31) / 32 * 2;
  const int kq = wave * 8 + 2 * l4;  // this lane's first k; its k of steps 2 t, 2 t + 1 are kq + 32 t and the next
  // Rows, columns and k past the edge are clamped into the matrices so that every load is unconditional;
  // what was read for a k past the edge is replaced by zero, results past the edge are not stored.
  const int64_t arow = (m0 + l15 < M) ? m0 + l15 : M - 1;
  const T* const Ap = AT ? P.A + arow : P.A + arow * P.lda;
  const int64_t astep = AT ? P.lda : 1;
  const T* Bp[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) Bp[j] = P.B + ((n0 + 16 * j + l15 < N) ? n0 + 16 * j + l15 : N - 1);

  using vec2_t = typename Mfma<T>::vec2_t;
  const bool pairs = !AT && K >= 2 && K % 2 == 0 && ((uintptr_t)P.A % (2 * sizeof(T)) == 0) && (P.lda % 2 == 0);  // uniform
  auto k_of = [&](int s) { return kq + 32 * (s >> 1) + (s & 1); };
  T a[SMAX], b[NB][SMAX];
  auto load_half = [&](auto hc) __attribute__((always_inline)) {
    constexpr int H = decltype(hc)::value;
    if (pairs) {
#pragma unroll
      for (int s = H * 16; s < H * 16 + 16; s += 2) {
        // the pair (k, k + 1); K is even here, so a pair is inside the row or wholly past it (then clamped, unused)
        const int k = k_of(s);
        const int64_t kc = k < K ? k : K - 2;
        const vec2_t v = *reinterpret_cast<const vec2_t*>(Ap + kc);
        a[s] = v[0];
        a[s + 1] = v[1];
      }
    } else {
#pragma unroll
      for (int s = H * 16; s < H * 16 + 16; ++s) {
        const int k = k_of(s);
        const int64_t kc = k < K ? k : K - 1;
        a[s] = Ap[kc * astep];
      }
    }
#pragma unroll
    for (int s = H * 16; s < H * 16 + 16; ++s) {
      const int k = k_of(s);
      const int64_t kc = k < K ? k : K - 1;
#pragma unroll
      for (int j = 0; j < NB; ++j) b[j][s] = Bp[j][kc * P.ldb];
    }
  };
  load_half(std::integral_constant<int, 0>{});
  if (SMAX == 32 && S > 16) load_half(std::integral_constant<int, 1>{});  // uniform
  T c[NB][4];
  if (wave == 0) {  // uniform
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int r = m0 + Mfma<T>::row_of(v, lane), cc = n0 + 16 * j + l15;
        const int64_t rc = r < M ? r : M - 1, ccl = cc < N ? cc : N - 1;
        c[j][v] = P.C[rc * P.ldc + ccl];
      }
  }
  acc_t acc[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) acc[j] = acc_t{0, 0, 0, 0};
  auto mul_half = [&](auto hc) __attribute__((always_inline)) {
    constexpr int H = decltype(hc)::value;
#pragma unroll
    for (int s = H * 16; s < H * 16 + 16; ++s) {
      const bool in = k_of(s) < K;
#pragma unroll
      for (int j = 0; j < NB; ++j) acc[j] = Mfma<T>::mma(in ? a[s] : T(0), in ? b[j][s] : T(0), acc[j]);
    }
  };
  mul_half(std::integral_constant<int, 0>{});
  if (SMAX == 32 && S > 16) mul_half(std::integral_constant<int, 1>{});  // uniform
  // partial blocks of waves 1..3: element v of lane l of column block j at ((wave - 1) * NB + j) * 256 + v * 64 + l
  if (wave > 0) {
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) red[((wave - 1) * NB + j) * 256 + v * 64 + lane] = acc[j][v];
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int at = j * 256 + v * 64 + lane;
        const T sum = ((acc[j][v] + red[at]) + red[NB * 256 + at]) + red[2 * NB * 256 + at];
        const T out = c[j][v] - sum;
        const int r = m0 + Mfma<T>::row_of(v, lane), cc = n0 + 16 * j + l15;
        if (r < M && cc < N) {
          P.C[(int64_t)r * P.ldc + cc] = out;
          if (P.C2) P.C2[(int64_t)r * P.ldc2 + cc] = out;
        }
      }
  }
}

// SMAX: steps per wave the kernel is built for (16 SMAX >= K of every product of the launch).
template <typename T, bool AT, int SMAX>
__global__ void __launch_bounds__(kSkinnyThreads) skinny_kernel(const SkinnyGroup<T> g) {
  static_assert(SMAX == 16 || SMAX == 32, "steps per wave");
  __shared__ T red[3 * 2 * 256];
  const int bid = (int)blockIdx.x;
  int pi = 0;
#pragma unroll
  for (int q = 1; q < kSkinnyMaxParts; ++q)
    if (q < g.nparts && bid >= g.part[q].tile_begin) pi = q;
  const SkinnyPart<T>& P = g.part[pi];
  if (P.wide) skinny_block<T, AT, 16, 2>(P, bid - P.tile_begin, red);  // uniform
  else skinny_block<T, AT, SMAX, 1>(P, bid - P.tile_begin, red);
}

}  // namespace dla
