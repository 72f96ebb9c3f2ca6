// Trailing-matrix update of the blocked factorisations, specialised for its shape:
//   LU:        A22 (m x m)       -= L21 (m x b) * U12 (b x m)
//   Cholesky:  lower(A22)        -= L21 * L21^T
// with b = block size <= 128, so the product is a rank-b update that streams the trailing matrix
// once (read + write) for 2*b flops per element: 16 flop/byte at b = 128 in fp64, just above the
// MFMA/HBM ridge.  The generic LDS-tiled GEMM re-stages both operands for every output tile and
// loads its C tile up front; here the left panel never moves:
//
//   - a workgroup (8 waves) owns 128 rows of L21; every wave keeps its 16 x b slice as MFMA
//     left-operand fragments IN REGISTERS (negated, so the accumulators can start from C);
//   - the workgroup then walks a range of column blocks of the trailing matrix, 32 or 64 columns
//     wide (NCB = 2 or 4 MFMA blocks; the wide form for large trailing matrices, whose rows are
//     then touched in 512-byte pieces, the narrow one where the wide one would leave compute units
//     without work): the b x cols block of the right operand is staged through double-buffered
//     LDS, the 16 x cols block of C per wave is prefetched into registers two iterations ahead,
//     32 * NCB MFMAs per wave and iteration run from registers + LDS, and the finished block is
//     stored while the next one computes.
//   - the eight waves form two groups of four (one wave of each group per SIMD) that take turns
//     on the MFMA pipes: while one group multiplies a column block, the other stores its previous
//     result, fetches its share of the next right-operand block and its next C block, and writes
//     the share to LDS; two barriers per block keep the groups in anti-phase.
//
// Two depths are instantiated (KMAX).  128: one panel of the factorisation, as above.  256: two
// panels at once, the form the factorisations use while the trailing matrix is large -- every
// element of C then carries 4*128 flops per read and write, 32 flop/byte, which takes the update
// off the memory bound.  The left panel then fills 128 registers per lane, so the column blocks
// are 16 wide in fp64 (NCB = 1: one accumulator block per wave and set; fp32 keeps NCB = 2); MFMAs per
// wave and iteration, right-operand bytes per iteration and the pipeline are the same as at depth 128
// with NCB = 2.
//
// Two forms of a work item (PLAIN): the general one, whose steps test whether a block exists, is ragged or
// belongs to the excluded leading block, and -- for a wave whose rows and an item whose blocks all lie inside
// the matrix at full depth -- one without a condition in its steps: buffer loads and stores (scalar base and
// offset, one constant per-lane offset), ends of the item and excluded blocks switched off through an
// out-of-range offset.  Only in straight-line code does the compiler count the loads in flight exactly; behind
// the general form's branches it waits for all of them before every use.
//
// Work list: (row panel, column range) items of roughly equal size, derived from blockIdx alone
// (update_kernel).  One launch cuts every row panel into whole work items, which leaves compute units
// idle when the panel count does not divide them well: an LU update is then given to two launches by
// rows (host side), and a large lower-triangular update to update_span_kernel, whose work items are
// equal runs of the column blocks of all panels and cross from one row panel into the next.
#pragma once
#include <type_traits>
#include "dla_common.hpp"

namespace dla {

constexpr int kUpdRows = 128;   // rows per workgroup (8 waves x 16 rows)
constexpr int kUpdThreads = 512;
constexpr int kUpdKMax = 128;   // largest block size b (depth of one panel)
// the forms that take the kernel instantiation with condition-free work items
template <typename T, bool LOWER>
constexpr bool kUpdPlainForm = true;

template <typename T>
struct UpdateArgs {
  const T* L;   // m x b left panel (L21)
  const T* R;   // LU: b x m right panel (U12);  Cholesky: the same m x b panel as L
  T* C;         // m x mc trailing matrix
  int64_t ld;   // common leading dimension (all three live in the same matrix)
  int m, b;     // rows of L and C; depth
  int mc;       // columns of C and of R: m, except for an LU launch that covers only part of the rows
  int bpi;      // target number of column blocks per work item
  int items;    // number of work items = grid size
  int skip;     // the leading skip x skip block of C (skip: multiple of 16) is not written: another stream owns it
};

template <typename T, bool LOWER, int NCB, int KMAX = kUpdKMax>
struct UpdateLds {
  // The b x cols right-operand block is stored in MFMA fragment order: element (k, col) sits at
  // ((k/4)*NCB + col/16)*64 + (k%4)*16 + col%16, i.e. the 64 values one wave reads for k-step k/4 and
  // column block col/16 are contiguous in lane order, so fragment reads are conflict free.
  static constexpr int B_ELEMS = KMAX * NCB * 16;
  static constexpr int B_PAD = B_ELEMS;
  // the left panel is staged through the same memory, 64 k-columns at a time: [rows][65]
  static constexpr int A_HALF = kUpdRows * 65;
  static constexpr int ELEMS = (2 * B_PAD > A_HALF) ? 2 * B_PAD : A_HALF;
  static constexpr int BYTES = ELEMS * (int)sizeof(T);
};

// column blocks (cols wide) row panel p (0-based) has to update, and the number of work items it is cut into
__host__ __device__ inline int update_blocks_of_panel(int p, int m, bool lower, int cols) {
  const int width = lower ? ((p + 1) * kUpdRows < m ? (p + 1) * kUpdRows : m) : m;
  return (width + cols - 1) / cols;
}
__host__ __device__ inline int update_items_of_panel(int p, int m, int bpi, bool lower, int cols) {
  return (update_blocks_of_panel(p, m, lower, cols) + bpi - 1) / bpi;
}

// One segment of a work item: the row panel `panel` against the column blocks col_begin,
// col_begin + col_step, ... whose first column lies below col_end.
template <typename T, bool LOWER, int NCB, int KMAX, bool PLAIN = false>
__device__ __forceinline__ void update_segment(const UpdateArgs<T>& g, T* const smem, const int panel, const int col_begin,
                                               const int col_step, const int col_end) {
  using acc_t = typename Mfma<T>::acc_t;
  using LD = UpdateLds<T, LOWER, NCB, KMAX>;
  constexpr int kUpdCols = NCB * 16;  // columns per iteration
  constexpr int KSTEPS = KMAX / 4;    // 32 or 64
  const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l15 = lane & 15, l4 = lane >> 4;
  const int m = g.m, b = g.b;
  const int mc = LOWER ? g.m : g.mc;  // column extent (the lower-triangular form is always square)
  const int64_t ld = g.ld;
  const int row0 = panel * kUpdRows;

  // ---- left panel -> registers (through LDS for coalesced global reads) -----------------------
  // 64 k-columns per pass; the loads of the next pass are issued before this pass goes through LDS, so the
  // passes cost one round trip to memory between them, not one each.
  T afrag[KSTEPS];
  const int wrow0 = row0 + wave * 16;  // first row of this wave
  constexpr int A_PASSES = KMAX / 64;
  T va[2][16];  // two staging sets: rows x 64 k-columns, thread -> (row, 2 adjacent columns), 8 rows apart
  const int a_cp = (tid & 31) * 2, a_r0 = tid >> 5;
  auto load_a = [&](int pass, T (&v)[16]) __attribute__((always_inline)) {
    constexpr int RPP = kUpdThreads / 32;
    static_assert(kUpdRows / RPP == 8, "staging registers");
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int r = a_r0 + it * RPP;
      const int gr = (row0 + r < m) ? row0 + r : m - 1;
      const int k0 = pass * 64 + a_cp, k1 = k0 + 1;
      const T* p = g.L + (int64_t)gr * ld;
      v[2 * it] = p[k0 < b ? k0 : b - 1];
      v[2 * it + 1] = p[k1 < b ? k1 : b - 1];
      if (!(row0 + r < m && k0 < b)) v[2 * it] = T(0);
      if (!(row0 + r < m && k1 < b)) v[2 * it + 1] = T(0);
    }
  };
  load_a(0, va[0]);
  // ---- right-operand block loader: b x 32 block starting at column j0 -> registers -> LDS ------
  // LU:       rows k of U12, cols contiguous columns: thread -> (k = tid / 4, cols / 4 columns)
  // Cholesky: rows j0..j0+cols-1 of L21, b contiguous k: thread -> (row = tid % cols, BPT k-values)
  constexpr int BPT = KMAX * kUpdCols / kUpdThreads;  // 8 or 16 elements per thread
  constexpr int TPK = kUpdThreads / KMAX;             // LU: threads that share one k-row of the block
  static_assert(TPK * BPT == kUpdCols && BPT <= 16 && 16 % BPT == 0, "right-operand staging");
  T bst[BPT];
  // A block that lies inside the matrix with the full depth b = KMAX: no conditions, and every address is a
  // base that is uniform over the wave (scalar registers) plus one per-lane byte offset that never changes.
  const uint32_t boff = !LOWER ? (uint32_t)(((int64_t)(tid / TPK) * ld + (tid % TPK) * BPT) * (int64_t)sizeof(T))
                               : (uint32_t)(((int64_t)(tid % kUpdCols) * ld + (tid / kUpdCols) * BPT) * (int64_t)sizeof(T));
  // Those loads and stores are buffer instructions: a resource in scalar registers (base and extent), a scalar
  // byte offset per instruction and the constant per-lane offset.  No 64-bit address is ever formed in vector
  // registers, which is what the register allocation of the steady-state loop needs: with flat addresses the
  // loop spilled address pairs (and a reload brings a wait for every load in flight back) or reused
  // accumulator registers whose stores were still reading them.
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  char* const Cs = reinterpret_cast<char*>(g.C + (int64_t)(row0 + wave_s * 16) * ld);  // this wave's 16 rows of C
  // Offsets at or above kOob lie outside every resource used here (extents stay below 2^31 bytes): the hardware
  // returns zero for such a load and drops such a store, which is how a step switches off a prefetch or a store
  // that has no block to go to without a branch in the instruction stream.
  constexpr uint32_t kOob = 0x80000000u;
  constexpr int kRsrcFlags = 0x00020000;  // raw 32-bit data format of gfx9-family resources, no swizzle: offsets are plain bytes
  const int64_t ext_c = ((int64_t)15 * ld + mc) * (int64_t)sizeof(T);
  // one right-operand block: LU: KMAX rows of kUpdCols columns;  lower-triangular form: kUpdCols rows of KMAX columns
  const int64_t ext_r = (!LOWER ? (int64_t)(KMAX - 1) * ld + kUpdCols : (int64_t)(kUpdCols - 1) * ld + KMAX) * (int64_t)sizeof(T);
  const bool ext_fit = ext_c < (int64_t)kOob && ext_r < (int64_t)kOob;
  const __amdgpu_buffer_rsrc_t rs_c = __builtin_amdgcn_make_buffer_rsrc(Cs, 0, ext_fit ? (int)ext_c : 0, kRsrcFlags);
  auto fetch_b_full = [&](int j0, bool on) __attribute__((always_inline)) {
    // the resource starts at the block, so that its extent does not grow with the matrix
    const T* const base = !LOWER ? g.R + j0 : g.R + (int64_t)j0 * ld;
    const __amdgpu_buffer_rsrc_t rs_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(base), 0, ext_fit ? (int)ext_r : 0, kRsrcFlags);
    const uint32_t vo = on ? boff : kOob;
    constexpr int PER = 16 / (int)sizeof(T);  // elements per 16-byte load
#pragma unroll
    for (int i = 0; i < BPT; i += PER) {
      const u32x4_t w = __builtin_amdgcn_raw_buffer_load_b128(rs_r, (int)(vo + i * (int)sizeof(T)), 0, 0);
      if constexpr (sizeof(T) == 8) {
        const double2_t d = __builtin_bit_cast(double2_t, w);
        bst[i] = d[0];
        bst[i + 1] = d[1];
      } else {
        const float4_t d = __builtin_bit_cast(float4_t, w);
        bst[i] = d[0];
        bst[i + 1] = d[1];
        bst[i + 2] = d[2];
        bst[i + 3] = d[3];
      }
    }
  };
  auto fetch_b = [&](int j0) {
    if (!LOWER) {
      const int k = tid / TPK, c0 = (tid % TPK) * BPT;
      const T* p = g.R + (int64_t)(k < b ? k : b - 1) * ld;
      const bool full = (j0 + kUpdCols <= mc) && (k < b);
      if (full) {
#pragma unroll
        for (int i = 0; i < BPT; ++i) bst[i] = p[j0 + c0 + i];
      } else {
#pragma unroll
        for (int i = 0; i < BPT; ++i) {
          const int c = j0 + c0 + i;
          const T x = p[c < mc ? c : mc - 1];
          bst[i] = (k < b && c < mc) ? x : T(0);
        }
      }
    } else {
      const int r = tid % kUpdCols, k0 = (tid / kUpdCols) * BPT;
      const int gr = (j0 + r < m) ? j0 + r : m - 1;
      const T* p = g.R + (int64_t)gr * ld;
      const bool full = (j0 + r < m) && (k0 + BPT <= b);
      if (full) {
#pragma unroll
        for (int i = 0; i < BPT; ++i) bst[i] = p[k0 + i];
      } else {
#pragma unroll
        for (int i = 0; i < BPT; ++i) {
          const int k = k0 + i;
          const T x = p[k < b ? k : b - 1];
          bst[i] = (j0 + r < m && k < b) ? x : T(0);
        }
      }
    }
  };
  auto stash_b = [&](int buf) {
    T* sb = smem + buf * LD::B_PAD;
    if (!LOWER) {
      const int k = tid / TPK, c0 = (tid % TPK) * BPT;  // BPT consecutive columns inside one 16-column block
      T* d = sb + ((k >> 2) * NCB + (c0 >> 4)) * 64 + (k & 3) * 16 + (c0 & 15);
#pragma unroll
      for (int i = 0; i < BPT; ++i) d[i] = bst[i];
    } else {
      const int col = tid % kUpdCols, k0 = (tid / kUpdCols) * BPT;  // BPT consecutive k of one column
#pragma unroll
      for (int i = 0; i < BPT; ++i) {
        const int k = k0 + i;
        sb[((k >> 2) * NCB + (col >> 4)) * 64 + (k & 3) * 16 + (col & 15)] = bst[i];
      }
    }
  };
  // ---- C block of this wave: 16 rows x cols columns = NCB MFMA blocks ------------------------------
  T* const Cw = g.C + (int64_t)wrow0 * ld;
  // (row_of(v, lane) = row_of(v, 0) + row_of(0, lane): the first part is the same for all lanes)
  // (a wave whose rows all lie below the matrix takes part in the staging of the right operand only: its C offsets
  // are out of range from the start)
  const int wrow0_s = __builtin_amdgcn_readfirstlane(wrow0);
  const uint32_t coff = wrow0_s >= m ? kOob : (uint32_t)(((int64_t)Mfma<T>::row_of(0, lane) * ld + l15) * (int64_t)sizeof(T));
  auto fetch_c_full = [&](acc_t (&c)[NCB], int j0, bool on) __attribute__((always_inline)) {
    const uint32_t vo = on ? coff : kOob;
#pragma unroll
    for (int q = 0; q < NCB; ++q)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const uint32_t so = ((uint32_t)Mfma<T>::row_of(v, 0) * (uint32_t)ld + (uint32_t)(j0 + q * 16)) * (uint32_t)sizeof(T);
        if constexpr (sizeof(T) == 8) c[q][v] = __builtin_bit_cast(double, __builtin_amdgcn_raw_buffer_load_b64(rs_c, (int)vo, (int)so, 0));
        else c[q][v] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_c, (int)vo, (int)so, 0));
      }
  };
  auto store_c_full = [&](const acc_t (&c)[NCB], int j0, bool on) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < NCB; ++q) {
      // (the excluded leading block: a condition that is uniform over the wave, per 16 columns)
      const uint32_t vo = (on && !(wrow0_s < g.skip && j0 + q * 16 < g.skip)) ? coff : kOob;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const uint32_t so = ((uint32_t)Mfma<T>::row_of(v, 0) * (uint32_t)ld + (uint32_t)(j0 + q * 16)) * (uint32_t)sizeof(T);
        if constexpr (sizeof(T) == 8) __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2_t, (double)c[q][v]), rs_c, (int)vo, (int)so, 0);
        else __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, (float)c[q][v]), rs_c, (int)vo, (int)so, 0);
      }
    }
  };
  auto fetch_c = [&](acc_t (&c)[NCB], int j0) {
    const bool full = (wrow0 + 16 <= m) && (j0 + kUpdCols <= mc);
    if (full) {
#pragma unroll
      for (int q = 0; q < NCB; ++q)
#pragma unroll
        for (int v = 0; v < 4; ++v) c[q][v] = Cw[(int64_t)Mfma<T>::row_of(v, lane) * ld + j0 + q * 16 + l15];
    } else {
#pragma unroll
      for (int q = 0; q < NCB; ++q)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int r = Mfma<T>::row_of(v, lane), cc = j0 + q * 16 + l15;
          const int rc = (wrow0 + r < m) ? r : m - 1 - wrow0;  // row index stays inside the matrix
          const T x = Cw[(int64_t)rc * ld + (cc < mc ? cc : mc - 1)];
          c[q][v] = (wrow0 + r < m && cc < mc) ? x : T(0);
        }
    }
  };
  auto store_c = [&](const acc_t (&c)[NCB], int j0) {
    const bool full = (wrow0 + 16 <= m) && (j0 + kUpdCols <= mc);
#pragma unroll
    for (int q = 0; q < NCB; ++q) {
      if (wrow0 < g.skip && j0 + q * 16 < g.skip) continue;  // uniform per wave: the excluded leading block
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int r = Mfma<T>::row_of(v, lane), cc = j0 + q * 16 + l15;
        if (full || (wrow0 + r < m && cc < mc)) Cw[(int64_t)r * ld + cc] = c[q][v];
      }
    }
  };
  auto multiply = [&](acc_t (&c)[NCB], int buf) {
    const T* sb = smem + buf * LD::B_PAD + lane;
    T f[NCB], nx[NCB];
#pragma unroll
    for (int q = 0; q < NCB; ++q) f[q] = sb[q * 64];
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
#pragma unroll
      for (int q = 0; q < NCB; ++q)  // fragments of the next k-step are requested before this step's MFMAs issue
        nx[q] = (kk + 1 < KSTEPS) ? sb[((kk + 1) * NCB + q) * 64] : T(0);
#pragma unroll
      for (int q = 0; q < NCB; ++q) c[q] = Mfma<T>::mma(afrag[kk], f[q], c[q]);
#pragma unroll
      for (int q = 0; q < NCB; ++q) f[q] = nx[q];
    }
  };
  // ---- pipeline over the column blocks, the two wave groups in anti-phase -------------------------
  //   barrier X_j : block j of the right operand is complete in LDS buffer buf, buffer buf^1 is free
  //   slot 1      : group 0 multiplies block j | group 1 stores its block j-1, fetches for j+1, fills its share of buf^1
  //   barrier Y_j
  //   slot 2      : group 1 multiplies block j | group 0 stores its block j,   fetches for j+1, fills its share of buf^1
  const int grp = wave >> 2;
  // the part of a block step that does not need the MFMA pipe
  // Prefetch distances: the right-operand share in bst is fetched one whole block step before it is
  // written to LDS, and a C block is fetched two steps before it is multiplied (three accumulator
  // sets rotate), so neither the LDS write nor the first MFMA of a step waits on a fresh load.
  auto side_work = [&](acc_t (&done)[NCB], int jdone, bool have_done, acc_t (&tgt)[NCB], int jc, int buf) {
    const int jn = jc + col_step, jnn = jc + 2 * col_step;
    if (jn < col_end) stash_b(buf ^ 1);  // block jn, fetched during the previous step
    if (jnn < col_end) fetch_b(jnn);     // block after that
    if (have_done) store_c(done, jdone);
    if (jnn < col_end) fetch_c(tgt, jnn);
  };
  acc_t c0[NCB], c1[NCB], c2[NCB];
  // ---- the whole work item without a condition in its steps ------------------------------------------------
  // For a wave whose rows, and a work item all of whose blocks, lie inside the matrix and outside the excluded
  // leading block (full depth b = KMAX): in straight-line code the compiler counts the loads in flight exactly
  // (a C block is used two steps after its loads, behind twelve younger loads and stores), where the branches
  // of the general form make it wait for every load before every use, which turns the prefetches into round
  // trips.  What the ends of the item need -- no store before the first block has been multiplied, no prefetch
  // behind the last block -- is switched off through the offset (kOob), not by a branch.  The steps come three
  // to a loop iteration (one rotation of the accumulator sets) and one or two more behind the loop.  Barriers
  // and LDS protocol are those of the general form below, step for step, so the waves of a workgroup may take
  // different forms.  (Barrier Y protects no data, it keeps the wave groups in anti-phase; without it the large
  // updates are 3-10 % slower: measured.)
  const int cb = __builtin_amdgcn_readfirstlane(col_begin), cs = __builtin_amdgcn_readfirstlane(col_step);
  const int ce = __builtin_amdgcn_readfirstlane(col_end);
  const int nblk = (ce - cb + cs - 1) / cs;  // blocks of this item
  const bool item_plain = PLAIN && __builtin_amdgcn_readfirstlane((int)((wrow0 + 16 <= m || wrow0 >= m) && (b == KMAX) && ext_fit &&
                                                                        (cb + (nblk - 1) * cs + kUpdCols <= mc)));
  if constexpr (PLAIN) {
    if (item_plain) {  // the first block's operands are on their way while the left panel goes through LDS
      fetch_b_full(cb, true);
      fetch_c_full(c0, cb, true);
    }
  }
#pragma unroll
  for (int pass = 0; pass < A_PASSES; ++pass) {
    if (pass + 1 < A_PASSES) load_a(pass + 1, va[(pass + 1) & 1]);
    {
      constexpr int RPP = kUpdThreads / 32;
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int r = a_r0 + it * RPP;
        smem[r * 65 + a_cp] = -va[pass & 1][2 * it];
        smem[r * 65 + a_cp + 1] = -va[pass & 1][2 * it + 1];
      }
    }
    lds_barrier();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) afrag[pass * 16 + kk] = smem[(wave * 16 + l15) * 65 + kk * 4 + l4];
    lds_barrier();
  }
  if constexpr (PLAIN) {
    if (item_plain) {
      const int grp_s = __builtin_amdgcn_readfirstlane(wave >> 2);
      auto step0 = [&](acc_t (&cur)[NCB], acc_t (&tgt)[NCB], int jc_, int b_) __attribute__((always_inline)) {
        const int jnn = jc_ + 2 * cs;
        const bool prefetch = jnn < ce;
        multiply(cur, b_);
        lds_barrier();  // Y
        stash_b(b_ ^ 1);
        fetch_b_full(jnn, prefetch);
        store_c_full(cur, jc_, true);
        fetch_c_full(tgt, jnn, prefetch);
        lds_barrier();  // X
      };
      auto step1 = [&](acc_t (&cur)[NCB], acc_t (&tgt)[NCB], int jc_, int b_, bool store) __attribute__((always_inline)) {
        const int jnn = jc_ + 2 * cs;
        const bool prefetch = jnn < ce;
        stash_b(b_ ^ 1);
        fetch_b_full(jnn, prefetch);
        store_c_full(tgt, jc_ - cs, store);  // the previous block's result
        fetch_c_full(tgt, jnn, prefetch);
        lds_barrier();  // Y
        multiply(cur, b_);
        lds_barrier();  // X
      };
      int jc = cb, left = nblk, bf = 0;
      stash_b(0);
      fetch_b_full(jc + cs, left > 1);
      fetch_c_full(c1, jc + cs, left > 1);
      lds_barrier();
      if (grp_s == 0) {
        while (left >= 3) {
          step0(c0, c2, jc, bf);
          step0(c1, c0, jc + cs, bf ^ 1);
          step0(c2, c1, jc + 2 * cs, bf);
          bf ^= 1;
          jc += 3 * cs;
          left -= 3;
        }
        if (left >= 1) step0(c0, c2, jc, bf);
        if (left == 2) step0(c1, c0, jc + cs, bf ^ 1);
      } else {
        bool started = false;
        while (left >= 3) {
          step1(c0, c2, jc, bf, started);
          step1(c1, c0, jc + cs, bf ^ 1, true);
          step1(c2, c1, jc + 2 * cs, bf, true);
          started = true;
          bf ^= 1;
          jc += 3 * cs;
          left -= 3;
        }
        if (left == 0) {
          store_c_full(c2, jc - cs, true);
        } else {
          step1(c0, c2, jc, bf, started);
          if (left == 2) {
            step1(c1, c0, jc + cs, bf ^ 1, true);
            store_c_full(c1, jc + cs, true);
          } else {
            store_c_full(c0, jc, true);
          }
        }
      }
      return;
    }
  }
  // ---- the general form ------------------------------------------------------------------------------------
  fetch_b(col_begin);
  fetch_c(c0, col_begin);
  stash_b(0);
  if (col_begin + col_step < col_end) {
    fetch_b(col_begin + col_step);
    fetch_c(c1, col_begin + col_step);
  }
  lds_barrier();
  int buf = 0;
  // One block step.  cur holds this block's C; tgt is the set that becomes free in this step and
  // receives the C block two steps ahead.  Group 0 frees cur's predecessor itself (it stores right
  // after multiplying); for group 1 the previous block's result still sits in tgt when the step begins.
  auto block_step = [&](acc_t (&cur)[NCB], acc_t (&tgt)[NCB], int jp, int jc, bool first, int b_) {
    if (grp == 0) {
      multiply(cur, b_);
      lds_barrier();  // Y
      side_work(cur, jc, true, tgt, jc, b_);
      lds_barrier();  // X
    } else {
      side_work(tgt, jp, !first, tgt, jc, b_);
      lds_barrier();  // Y
      multiply(cur, b_);
      lds_barrier();  // X
    }
  };
  int jp = col_begin, jc = col_begin;
  bool first = true;
  for (;;) {
    block_step(c0, c2, jp, jc, first, buf);
    buf ^= 1;
    first = false;
    jp = jc;
    jc += col_step;
    if (jc >= col_end) {
      if (grp == 1) store_c(c0, jp);
      break;
    }
    block_step(c1, c0, jp, jc, false, buf);
    buf ^= 1;
    jp = jc;
    jc += col_step;
    if (jc >= col_end) {
      if (grp == 1) store_c(c1, jp);
      break;
    }
    block_step(c2, c1, jp, jc, false, buf);
    buf ^= 1;
    jp = jc;
    jc += col_step;
    if (jc >= col_end) {
      if (grp == 1) store_c(c2, jp);
      break;
    }
  }
}

template <typename T, bool LOWER, int NCB, int KMAX = kUpdKMax, bool PLAIN = false>
__global__ void __launch_bounds__(kUpdThreads) update_kernel(const UpdateArgs<T> g) {
  static_assert(KMAX % 64 == 0 && kUpdThreads % KMAX == 0, "depth");
  constexpr int kUpdCols = NCB * 16;  // columns per iteration
  extern __shared__ __align__(16) unsigned char smem_raw[];
  T* const smem = reinterpret_cast<T*>(smem_raw);
  const int m = g.m;
  const int mc = LOWER ? g.m : g.mc;  // column extent (the lower-triangular form is always square)

  // ---- which work item: (row panel, first column, one-past-last column) ----------------------
  const int npanels = (m + kUpdRows - 1) / kUpdRows;
  int item = xcd_contiguous_id((int)blockIdx.x, g.items);
  int panel = 0, cnt = 0;
  for (;;) {
    cnt = update_items_of_panel(panel, LOWER ? m : mc, g.bpi, LOWER, kUpdCols);
    if (item < cnt || panel + 1 >= npanels) break;
    item -= cnt;
    ++panel;
  }
  // The panel's column blocks are dealt round-robin to its items: item q takes blocks q, q + cnt,
  // q + 2*cnt, ...  Items run side by side, so at any moment the items of one panel touch a run of
  // adjacent 256-byte pieces of the same matrix rows (DRAM page locality), and every panel is at
  // about the same right-operand block (L2 reuse).
  const int nblocks = update_blocks_of_panel(panel, LOWER ? m : mc, LOWER, kUpdCols);
  const int width = LOWER ? ((panel + 1) * kUpdRows < m ? (panel + 1) * kUpdRows : m) : mc;
  const int col_begin = item * kUpdCols;         // first block of this item
  const int col_step = cnt * kUpdCols;           // distance between its blocks
  const int col_end = width;                     // a block is valid while its first column is < width
  (void)nblocks;
  if (col_begin >= col_end) return;  // uniform

  update_segment<T, LOWER, NCB, KMAX, PLAIN>(g, smem, panel, col_begin, col_step, col_end);
}

// The same update with work items of exactly equal size for the lower-triangular form, whose row
// panels hold 1 .. m/128 times as many column blocks: the column blocks of all panels, panel after
// panel, are cut into gridDim.x equal runs, and a workgroup walks its run, reloading the left panel
// where the run crosses into the next row panel.  (Per-panel items, as above, leave a quarter of the
// compute units idle on a large trapezoid: a small panel's item is a fraction of a large panel's.)
template <typename T, int NCB, int KMAX = kUpdKMax, bool PLAIN = false>
__global__ void __launch_bounds__(kUpdThreads) update_span_kernel(const UpdateArgs<T> g, const int64_t total_blocks) {
  constexpr int kUpdCols = NCB * 16;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  T* const smem = reinterpret_cast<T*>(smem_raw);
  const int m = g.m;
  const int npanels = (m + kUpdRows - 1) / kUpdRows;
  const int item = xcd_contiguous_id((int)blockIdx.x, (int)gridDim.x);
  int64_t lo = ((int64_t)item * total_blocks) / (int64_t)gridDim.x;
  int64_t left = ((int64_t)(item + 1) * total_blocks) / (int64_t)gridDim.x - lo;  // blocks of this item
  int panel = 0;
  while (panel + 1 < npanels && lo >= update_blocks_of_panel(panel, m, true, kUpdCols)) {
    lo -= update_blocks_of_panel(panel, m, true, kUpdCols);
    ++panel;
  }
  while (left > 0 && panel < npanels) {  // uniform over the workgroup
    const int here = update_blocks_of_panel(panel, m, true, kUpdCols);
    const int64_t take = left < here - lo ? left : here - lo;
    const int width = (panel + 1) * kUpdRows < m ? (panel + 1) * kUpdRows : m;
    const int end = (int)(lo + take) * kUpdCols;
    update_segment<T, true, NCB, KMAX, PLAIN>(g, smem, panel, (int)lo * kUpdCols, kUpdCols, end < width ? end : width);
    lds_barrier();  // the next segment restages the left panel through the same memory
    left -= take;
    lo = 0;
    ++panel;
  }
}

}  // namespace dla
