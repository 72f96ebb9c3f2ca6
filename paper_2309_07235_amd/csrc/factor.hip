// Host drivers of the blocked right-looking factorisations: for every block
// column  (1) factor the diagonal block, (2) solve the panels, (3) update the
// trailing matrix with the MFMA GEMM (the step that dominates the run time).
#include "factor_kernels.hpp"
#include "update_kernel.hpp"
#include "host_common.hpp"

namespace dla {

static inline size_t round_up_sz(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Workspace: two parity sets of {inverted lower sub-blocks, inverted upper sub-blocks}.
static size_t inv_set_bytes(dla_dtype dt) {
  return round_up_sz((size_t)(kNbMax / kIb) * 256 * (dt == DLA_F64 ? 8 : 4), 256);
}

size_t factor_workspace_bytes_impl(int64_t n, dla_dtype dt, const dla_factor_params* p) {
  (void)n;
  (void)p;
  return 4 * inv_set_bytes(dt);
}

int resolve_factor_params(dla_dtype dt, int64_t n, const dla_factor_params* in, int op, int* nb, int* lookahead,
                          GemmSchedule* upd) {
  (void)n;
  int b = in ? in->nb : 0;
  if (b == 0) b = 128;
  if (b < 16 || b > kNbMax || b % 16 != 0) return DLA_ERR_UNSUPPORTED_PARAMS;
  int la = in ? in->lookahead : -1;
  if (la < -1 || la > 1) return DLA_ERR_UNSUPPORTED_PARAMS;
  if (la == -1) la = 1;
  *nb = b;
  *lookahead = la;
  return resolve_schedule(dt, in ? &in->update : nullptr, op, upd);
}

template <typename T, int KIND>
static int launch_diag(const DiagArgs<T>& a, hipStream_t st) {
  auto kern = diag_kernel<T, KIND>;
  static bool attr_done = false;
  if (!attr_done) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            diag_lds_bytes<T>()) != hipSuccess)
      return DLA_ERR_HIP;
    attr_done = true;
  }
  ProfileScope scope(PHASE_DIAG, 0.0, st);
  hipLaunchKernelGGL(kern, dim3(1), dim3(kDiagThreads), diag_lds_bytes<T>(), st, a);
  return hipGetLastError() == hipSuccess ? DLA_SUCCESS : DLA_ERR_HIP;
}

// Rank-b trailing update with the panel-stationary kernel (see update_kernel.hpp).
template <typename T, int KIND>
static int launch_update(const T* L, const T* R, T* C, int64_t ld, int64_t m, int b, hipStream_t st) {
  if (m <= 0) return DLA_SUCCESS;
  constexpr bool LOWER = (KIND == KIND_CHOL);
  auto kern = update_kernel<T, LOWER>;
  using LD = UpdateLds<T, LOWER>;
  static bool attr_done = false;
  if (!attr_done) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            LD::BYTES) != hipSuccess)
      return DLA_ERR_HIP;
    attr_done = true;
  }
  UpdateArgs<T> a;
  a.L = L;
  a.R = R;
  a.C = C;
  a.ld = ld;
  a.m = (int)m;
  a.b = b;
  const int npanels = (int)((m + kUpdRows - 1) / kUpdRows);
  int64_t total_blocks = 0;
  for (int p = 0; p < npanels; ++p) total_blocks += update_blocks_of_panel(p, (int)m, LOWER);
  // one 8-wave workgroup per compute unit: aim at one full round of at most 256 items
  const int slots = 256;
  a.bpi = (int)((total_blocks + slots - 1) / slots);
  if (a.bpi < 1) a.bpi = 1;
  int items = 0;
  for (;;) {
    items = 0;
    for (int p = 0; p < npanels; ++p) items += update_items_of_panel(p, (int)m, a.bpi, LOWER);
    if (items <= slots || a.bpi >= (1 << 20)) break;
    ++a.bpi;  // rounding up per panel overshot the slot count
  }
  a.items = items;
  const double flops = (LOWER ? 1.0 : 2.0) * (double)m * (double)m * (double)b;
  ProfileScope scope(PHASE_GEMM, flops, st);
  hipLaunchKernelGGL(kern, dim3((unsigned)items), dim3(kUpdThreads), LD::BYTES, st, a);
  return hipGetLastError() == hipSuccess ? DLA_SUCCESS : DLA_ERR_HIP;
}

template <typename T, int KIND>
static int launch_trsm(TrsmArgs<T> a, hipStream_t st) {
  auto kern = trsm_kernel<T, KIND>;
  static bool attr_done = false;
  if (!attr_done) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            trsm_lds_bytes<T>()) != hipSuccess)
      return DLA_ERR_HIP;
    attr_done = true;
  }
  const int per_wg = (kTrsmThreads / 64) * kIb;  // panel rows/columns one workgroup solves
  const int wgs = (a.m + per_wg - 1) / per_wg;
  a.n_left = (KIND == KIND_LU) ? wgs : 0;
  const int grid = a.n_left + wgs;
  if (grid <= 0) return DLA_SUCCESS;
  ProfileScope scope(PHASE_TRSM, 0.0, st);
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kTrsmThreads), trsm_lds_bytes<T>(), st, a);
  return hipGetLastError() == hipSuccess ? DLA_SUCCESS : DLA_ERR_HIP;
}

// Helper stream and events for look-ahead: library-owned, default priority, created on first use
// and kept for the life of the process.
struct LookaheadCtx {
  hipStream_t helper = nullptr;
  hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
  bool ok = false;
};
static LookaheadCtx& lookahead_ctx() {
  static LookaheadCtx ctx;
  if (!ctx.ok) {
    bool good = hipStreamCreateWithFlags(&ctx.helper, hipStreamNonBlocking) == hipSuccess;
    for (int i = 0; i < 4 && good; ++i) good = hipEventCreateWithFlags(&ctx.ev[i], hipEventDisableTiming) == hipSuccess;
    ctx.ok = good;
  }
  return ctx;
}

// Schedule of the small look-ahead panel updates (skinny products with k = nb): small tiles, so a
// panel that is only a few hundred rows long still spreads over many compute units.
static GemmSchedule panel_schedule() { return GemmSchedule{32, 32, 16, 4, 16, 16}; }

template <typename T, int KIND>
static int factor_impl(T* A, int64_t n, int64_t lda, const dla_factor_params* p, void* ws, size_t ws_bytes,
                       hipStream_t st, int* d_info) {
  const dla_dtype dt = sizeof(T) == 8 ? DLA_F64 : DLA_F32;
  int nb, lookahead;
  GemmSchedule upd;
  const int op = (KIND == KIND_LU) ? OP_SUB : OP_SUB_NT_LOWER;
  int rc = resolve_factor_params(dt, n, p, op, &nb, &lookahead, &upd);
  if (rc != DLA_SUCCESS) return rc;
  if (n == 0) return DLA_SUCCESS;
  if (!ws || ws_bytes < factor_workspace_bytes_impl(n, dt, p) || ((uintptr_t)ws % 256)) return DLA_ERR_WORKSPACE;
  const bool auto_tile = !(p && (p->update.tile_m != 0 || p->update.tile_n != 0));

  unsigned char* wsb = static_cast<unsigned char*>(ws);
  const size_t set = inv_set_bytes(dt);
  auto inv_lo_of = [&](int step) { return reinterpret_cast<T*>(wsb + (size_t)(2 * (step & 1)) * set); };
  auto inv_up_of = [&](int step) { return reinterpret_cast<T*>(wsb + (size_t)(2 * (step & 1) + 1) * set); };

  // diagonal block + panel solves of the block column starting at k0, on stream s
  auto panel = [&](int64_t k0, int step, hipStream_t s) -> int {
    const int b = (int)((n - k0 < nb) ? n - k0 : nb);
    const int64_t m = n - k0 - b;
    T* const Akk = A + k0 * lda + k0;
    DiagArgs<T> da;
    da.A = Akk;
    da.lda = lda;
    da.b = b;
    da.k0 = (int)k0;
    da.info = d_info;
    da.inv_lo = inv_lo_of(step);
    da.inv_up = inv_up_of(step);
    int r = launch_diag<T, KIND>(da, s);
    if (r != DLA_SUCCESS || m == 0) return r;
    TrsmArgs<T> ta;
    ta.D = Akk;
    ta.left = Akk + b;                  // A12: b x m
    ta.right = Akk + (int64_t)b * lda;  // A21: m x b
    ta.lda = lda;
    ta.b = b;
    ta.m = (int)m;
    ta.n_left = 0;
    ta.inv_lo = da.inv_lo;
    ta.inv_up = da.inv_up;
    return launch_trsm<T, KIND>(ta, s);
  };
  // trailing-update schedule for an m x m update: the caller's, or by default small macro-tiles.
  // With k = nb the update streams the trailing matrix once (16 flop per byte at nb = 128), so
  // what matters is how well loads, MFMA and stores of many co-resident workgroups overlap;
  // measured on the update shape, 64 x 64 tiles win for large m and 32 x 32 below that.
  auto update_schedule = [&](int64_t m) {
    if (!auto_tile) return upd;
    GemmSchedule s = upd;
    if (KIND == KIND_LU && m >= 3000) {
      s.tm = s.tn = 64;
      s.wm = s.wn = 32;
    } else {
      s.tm = s.tn = 32;
      s.wm = s.wn = 16;
    }
    return s;
  };

  // m x m trailing update behind the panel whose L21 / U12 are given
  auto trailing = [&](const T* Lp, const T* Up, T* Cp, int64_t mm, int bb, hipStream_t s) -> int {
    if (auto_tile) return launch_update<T, KIND>(Lp, KIND == KIND_LU ? Up : Lp, Cp, lda, mm, bb, s);
    const GemmSchedule us = update_schedule(mm);
    if (KIND == KIND_LU) return run_gemm<T>(us, OP_SUB, Lp, lda, Up, lda, Cp, lda, mm, mm, bb, s);
    return run_gemm<T>(us, OP_SUB_NT_LOWER, Lp, lda, Lp, lda, Cp, lda, mm, mm, bb, s);
  };

  LookaheadCtx* ctx = nullptr;
  if (lookahead && n > 2 * (int64_t)nb) {
    ctx = &lookahead_ctx();
    if (!ctx->ok) return DLA_ERR_HIP;
  }

  // Look-ahead keeps the latency chain  diag(k) -> panel solves(k) -> strip update(k) -> diag(k+1)
  // back to back on the caller's stream; the bulk of every trailing update runs on the helper
  // stream.  "Strip k+1" is what the next panel needs: the next block column and block row of
  // the trailing matrix.  bulk(k) updates everything behind strip k+1 and may still be running
  // while panel k+1 is factored.  strip(k+1) touches memory bulk(k) writes, so it waits for it.
  hipEvent_t e_panel = ctx ? ctx->ev[0] : nullptr;  // recorded on the caller's stream after the panel solves
  hipEvent_t e_bulk = ctx ? ctx->ev[1] : nullptr;   // recorded on the helper stream after a bulk update
  bool bulk_pending = false;

  if ((rc = panel(0, 0, st)) != DLA_SUCCESS) return rc;
  int step = 0;
  for (int64_t k0 = 0; k0 < n; k0 += nb, ++step) {
    const int b = (int)((n - k0 < nb) ? n - k0 : nb);
    const int64_t m = n - k0 - b;
    if (m == 0) break;
    T* const Akk = A + k0 * lda + k0;
    T* const L21 = Akk + (int64_t)b * lda;  // m x b
    T* const U12 = Akk + b;                 // b x m   (LU)
    T* const A22 = L21 + b;
    const int64_t bn = m < nb ? m : nb;      // width of the next block column
    const int64_t mr = m - bn;               // what is left behind it
    if (ctx && mr > 0) {
      // bulk(k) on the helper stream: needs panel k (event) and, through stream order, bulk(k-1)
      if (hipEventRecord(e_panel, st) != hipSuccess || hipStreamWaitEvent(ctx->helper, e_panel, 0) != hipSuccess)
        return DLA_ERR_HIP;
      // strip(k) on the caller's stream: needs bulk(k-1), which wrote the same strip
      if (bulk_pending && hipStreamWaitEvent(st, e_bulk, 0) != hipSuccess) return DLA_ERR_HIP;
      const GemmSchedule ps = panel_schedule();
      if (KIND == KIND_LU) {
        GemmGroup<T> g;
        g.nprob = 2;
        g.prob[0] = make_problem<T>(ps, OP_SUB, L21, lda, U12, lda, A22, lda, m, bn, b, 0);  // block column
        const int t0 = problem_tiles(ps, OP_SUB, g.prob[0]);
        g.prob[1] = make_problem<T>(ps, OP_SUB, L21, lda, U12 + bn, lda, A22 + bn, lda, bn, mr, b, t0);  // block row
        g.total_tiles = t0 + problem_tiles(ps, OP_SUB, g.prob[1]);
        ProfileScope scope(PHASE_GEMM, 2.0 * (double)b * ((double)m * bn + (double)bn * mr), st);
        if ((rc = launch_gemm<T>(ps, OP_SUB, g, st)) != DLA_SUCCESS) return rc;
      } else {
        if ((rc = run_gemm<T>(ps, OP_SUB_NT, L21, lda, L21, lda, A22, lda, m, bn, b, st)) != DLA_SUCCESS) return rc;
      }
      T* const C = A22 + bn * lda + bn;
      if ((rc = trailing(L21 + bn * lda, U12 + bn, C, mr, b, ctx->helper)) != DLA_SUCCESS) return rc;
      if (hipEventRecord(e_bulk, ctx->helper) != hipSuccess) return DLA_ERR_HIP;
      bulk_pending = true;
      // next panel right behind the strip update, on the caller's stream
      if ((rc = panel(k0 + b, step + 1, st)) != DLA_SUCCESS) return rc;
    } else {
      if (bulk_pending) {  // join: the remaining steps run on the caller's stream only
        if (hipStreamWaitEvent(st, e_bulk, 0) != hipSuccess) return DLA_ERR_HIP;
        bulk_pending = false;
      }
      if ((rc = trailing(L21, U12, A22, m, b, st)) != DLA_SUCCESS) return rc;
      if ((rc = panel(k0 + b, step + 1, st)) != DLA_SUCCESS) return rc;
    }
  }
  if (bulk_pending && hipStreamWaitEvent(st, e_bulk, 0) != hipSuccess) return DLA_ERR_HIP;
  if (KIND == KIND_CHOL && n > 1) {
    hipLaunchKernelGGL(zero_upper_kernel<T>, dim3((unsigned)((n + 255) / 256), (unsigned)(n < 32768 ? n : 32768)),
                       dim3(256), 0, st, A, lda, (int)n);
    if (hipGetLastError() != hipSuccess) return DLA_ERR_HIP;
  }
  return DLA_SUCCESS;
}

template <typename T>
int lu_factor_impl(T* A, int64_t n, int64_t lda, const dla_factor_params* p, void* ws, size_t ws_bytes,
                   hipStream_t st, int* d_info) {
  return factor_impl<T, KIND_LU>(A, n, lda, p, ws, ws_bytes, st, d_info);
}
template <typename T>
int cholesky_factor_impl(T* A, int64_t n, int64_t lda, const dla_factor_params* p, void* ws, size_t ws_bytes,
                         hipStream_t st, int* d_info) {
  return factor_impl<T, KIND_CHOL>(A, n, lda, p, ws, ws_bytes, st, d_info);
}

template int lu_factor_impl<double>(double*, int64_t, int64_t, const dla_factor_params*, void*, size_t, hipStream_t,
                                    int*);
template int lu_factor_impl<float>(float*, int64_t, int64_t, const dla_factor_params*, void*, size_t, hipStream_t,
                                   int*);
template int cholesky_factor_impl<double>(double*, int64_t, int64_t, const dla_factor_params*, void*, size_t,
                                          hipStream_t, int*);
template int cholesky_factor_impl<float>(float*, int64_t, int64_t, const dla_factor_params*, void*, size_t,
                                         hipStream_t, int*);

}  // namespace dla
