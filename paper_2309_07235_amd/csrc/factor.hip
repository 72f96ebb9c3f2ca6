// Host drivers of the blocked right-looking factorisations: for every block
// column  (1) factor the diagonal block, (2) solve the panels, (3) update the
// trailing matrix with the MFMA GEMM (the step that dominates the run time).
#include "factor_kernels.hpp"
#include "update_kernel.hpp"
#include "head_kernel.hpp"
#include <mutex>
#include "host_common.hpp"

namespace dla {

constexpr int kNumCu = 256;   // compute units of an MI355X
// Compute units a bulk update leaves to the latency chain and the side path (panel solves, strips) that run beside
// it: 32, and 64 for the fp64 updates of kWideReserveMinRows to kWideReserveMaxRows rows, whose side path is what
// those steps of the call wait for.  Measured with the condition-free update kernel (the bulk update got faster,
// the kernels beside it did not): LU N = 4000 2.07 -> 1.96 ms, N = 6000 4.37 -> 4.17 ms; above about 5000 rows the
// bulk update is the longer side again (LU N = 8192: 8.77 ms with 64 units at every size, 8.62 with them below 5120
// rows only).  Cholesky gains with it once it also defers its bulk updates down to 2560 rows (N = 4000 1.64 -> 1.59,
// N = 6000 3.14 -> 2.97, N = 8192 5.59 -> 5.44 ms; neither change helps alone).  fp32, whose bulk update is twice
// as fast, loses with 64 (LU N = 8192 4 %); 80 units and more lose from N = 6000 on.
constexpr int kChainCu = 32, kChainCuWide = 64;
constexpr int64_t kWideReserveMinRows = 2048, kWideReserveMaxRows = 5120;
constexpr int kWideMinBlocks = 2;  // 64-column update blocks once every slot gets at least this many
// Trailing matrices of at least this many rows run their bulk updates two panels at a time (measured:
// below these sizes the step is bound by the latency chain and the deeper strips only lengthen it).
constexpr int64_t kDeferMinRowsLu = 2560, kDeferMinRowsChol = 2560, kDeferMinRowsCholF32 = 4096;
// Cholesky updates of at least this many rows use work items that cross row panels (measured: 3-18 %
// faster from 6000 rows on, slower below 4000; inside the pipeline it pays from about 8000 rows).
constexpr int64_t kSpanMinRows = 6144;

static inline size_t round_up_sz(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Workspace: two parity sets of {inverted lower sub-blocks, inverted upper sub-blocks}, then two
// parity sets of {copy of the row-panel head, copy of the column-panel head} (kNbMax x kNbMax each).
static size_t inv_set_bytes(dla_dtype dt) {
  return round_up_sz((size_t)(kNbMax / kIb) * 256 * (dt == DLA_F64 ? 8 : 4), 256);
}
static size_t head_copy_bytes(dla_dtype dt) { return (size_t)kNbMax * kNbMax * (dt == DLA_F64 ? 8 : 4); }

size_t factor_workspace_bytes_impl(int64_t n, dla_dtype dt, const dla_factor_params* p) {
  (void)n;
  (void)p;
  return 4 * inv_set_bytes(dt) + 4 * head_copy_bytes(dt) + 256;  // + the hand-over counters of the latency chain
}

int resolve_factor_params(dla_dtype dt, int64_t n, const dla_factor_params* in, int op, FactorPlan* plan,
                          GemmSchedule* upd) {
  (void)n;
  int b = in ? in->nb : 0;
  if (b == 0) b = 128;
  const bool one_level = b >= 16 && b <= kNbMax && b % 16 == 0;
  const bool two_level = b > kNbMax && b <= 2 * kNbMax && b % 32 == 0;
  if (!one_level && !two_level) return DLA_ERR_UNSUPPORTED_PARAMS;
  int la = in ? in->lookahead : -1;
  if (la < -1 || la > 2) return DLA_ERR_UNSUPPORTED_PARAMS;
  if (la == -1) la = 1;
  const int defer = in ? in->defer_min_rows : 0;
  if (defer < -1) return DLA_ERR_UNSUPPORTED_PARAMS;
  const bool tiled = in && (in->update.tile_m != 0 || in->update.tile_n != 0 || in->update.tile_k != 0 ||
                            in->update.unroll_k != 0 || in->update.wave_m != 0 || in->update.wave_n != 0);
  // two sub-panels per panel need the pipeline's deferred bulk update and the kernel that takes depth 256
  if (two_level && (la == 0 || tiled)) return DLA_ERR_UNSUPPORTED_PARAMS;
  plan->nb_outer = b;
  plan->nb = two_level ? b / 2 : b;
  plan->lookahead = la;
  plan->two_level = two_level || (b == kNbMax && defer != -1 && !tiled);
  plan->defer_min_rows = two_level ? 0 : (defer > 0 ? defer : (op == OP_SUB ? kDeferMinRowsLu : (dt == DLA_F64 ? kDeferMinRowsChol : kDeferMinRowsCholF32)));
  return resolve_schedule(dt, in ? &in->update : nullptr, op, upd);
}

// Launch with an optional completion event: the event rides on the kernel's own dispatch packet
// instead of a separate marker packet behind it, which shortens the hand-over to a waiting stream.
template <typename K, typename A>
static inline void launch_ev(K kern, dim3 grid, dim3 block, int lds, hipStream_t st, hipEvent_t done, const A& a) {
  if (done) hipExtLaunchKernelGGL(kern, grid, block, lds, st, nullptr, done, 0, a);
  else hipLaunchKernelGGL(kern, grid, block, lds, st, a);
}

template <typename T, int KIND>
static int launch_diag(const DiagArgs<T>& a, hipStream_t st, hipEvent_t done = nullptr) {
  auto kern = diag_kernel<T, KIND>;
  static LdsLimitOnce lds_limit;
  if (!lds_limit.ensure(reinterpret_cast<const void*>(kern), diag_lds_bytes<T>())) return DLA_ERR_HIP;
  ProfileScope scope(PHASE_DIAG, 0.0, st);
  launch_ev(kern, dim3(1), dim3(kDiagThreads), diag_lds_bytes<T>(), st, done, a);
  return launch_status(__func__);
}

// Rank-b trailing update with the panel-stationary kernel (see update_kernel.hpp): one launch over
// the rows [0, m) of L and C and the columns [0, mc) of C (mc = m except for a launch that covers
// only part of the rows of an LU update).
template <typename T, int KIND, int NCB, int KMAX>
static int launch_update_rows(const T* L, const T* R, T* C, int64_t ld, int64_t m, int64_t mc, int b, int skip, int slots,
                              hipStream_t st, hipEvent_t done) {
  constexpr bool LOWER = (KIND == KIND_CHOL);
  constexpr int COLS = NCB * 16;
  void (*kern)(UpdateArgs<T>) = update_kernel<T, LOWER, NCB, KMAX>;
  using LD = UpdateLds<T, LOWER, NCB, KMAX>;
  static LdsLimitOnce lds_limit;
  if (!lds_limit.ensure(reinterpret_cast<const void*>(kern), LD::BYTES)) return DLA_ERR_HIP;
  UpdateArgs<T> a;
  a.L = L;
  a.R = R;
  a.C = C;
  a.ld = ld;
  a.m = (int)m;
  a.mc = (int)mc;
  a.b = b;
  a.skip = skip;
  const int npanels = (int)((m + kUpdRows - 1) / kUpdRows);
  int64_t total_blocks = 0;
  for (int p = 0; p < npanels; ++p) total_blocks += update_blocks_of_panel(p, (int)mc, LOWER, COLS);
  const double flops = (LOWER ? 1.0 : 2.0) * ((double)m * (double)mc - (double)skip * (double)skip) * (double)b;
  if constexpr (LOWER) {
    // a large trapezoid: work items of equal size that cross row panels (see update_span_kernel)
    if (m >= kSpanMinRows && total_blocks >= 8 * (int64_t)slots) {
      auto span = update_span_kernel<T, NCB, KMAX, kUpdPlainForm<T, true>>;
      static LdsLimitOnce span_lds_limit;
      if (!span_lds_limit.ensure(reinterpret_cast<const void*>(span), LD::BYTES)) return DLA_ERR_HIP;
      a.bpi = 1;
      a.items = slots;
      hipEvent_t p0 = nullptr, p1 = nullptr;
      if (profile_kernel_events(PHASE_UPDATE, flops, &p0, &p1)) {
        hipExtLaunchKernelGGL(span, dim3((unsigned)slots), dim3(kUpdThreads), LD::BYTES, st, p0, p1, 0, a, total_blocks);
        if (launch_status(__func__) != DLA_SUCCESS) return DLA_ERR_HIP;
        if (done && hip_note(hipEventRecord(done, st), "hipEventRecord") != 0) return DLA_ERR_HIP;
        return DLA_SUCCESS;
      }
      if (done) hipExtLaunchKernelGGL(span, dim3((unsigned)slots), dim3(kUpdThreads), LD::BYTES, st, nullptr, done, 0, a, total_blocks);
      else hipLaunchKernelGGL(span, dim3((unsigned)slots), dim3(kUpdThreads), LD::BYTES, st, a, total_blocks);
      return launch_status(__func__);
    }
  }
  // one 8-wave workgroup fits per compute unit: aim at one round of at most `slots` items
  a.bpi = (int)((total_blocks + slots - 1) / slots);
  if (a.bpi < 1) a.bpi = 1;
  int items = 0;
  for (;;) {
    items = 0;
    for (int p = 0; p < npanels; ++p) items += update_items_of_panel(p, (int)mc, a.bpi, LOWER, COLS);
    if (items <= slots || a.bpi >= (1 << 20)) break;
    ++a.bpi;  // rounding up per panel overshot the slot count
  }
  a.items = items;
  // the instantiation whose work items run without a condition in their steps where they lie inside the matrix
  if constexpr (kUpdPlainForm<T, LOWER>) {
    kern = update_kernel<T, LOWER, NCB, KMAX, true>;
    static LdsLimitOnce plain_lds_limit;
    if (!plain_lds_limit.ensure(reinterpret_cast<const void*>(kern), LD::BYTES)) return DLA_ERR_HIP;
  }
  hipEvent_t p0 = nullptr, p1 = nullptr;
  if (profile_kernel_events(PHASE_UPDATE, flops, &p0, &p1)) {
    // profiling: the dispatch carries the profiler's start / stop events, the completion event follows it
    hipExtLaunchKernelGGL(kern, dim3((unsigned)items), dim3(kUpdThreads), LD::BYTES, st, p0, p1, 0, a);
    if (launch_status(__func__) != DLA_SUCCESS) return DLA_ERR_HIP;
    if (done && hip_note(hipEventRecord(done, st), "hipEventRecord") != 0) return DLA_ERR_HIP;
    return DLA_SUCCESS;
  }
  launch_ev(kern, dim3((unsigned)items), dim3(kUpdThreads), LD::BYTES, st, done, a);
  return launch_status(__func__);
}

// All row panels of an LU update hold the same number of column blocks, so one launch cuts each into
// the same number c of work items and uses c * panels of the `slots` compute units: 126 panels on
// 224 units run at c = 1, on 56 % of the units.  Where that leaves more than a tenth of them idle, the
// rows go in two launches, back to back, that each fill the units: the first floor(slots / (c + 1))
// panels at c + 1 items per panel, the remaining few panels at as many items per panel as fit.
template <typename T, int KIND, int NCB, int KMAX = kUpdKMax>
static int launch_update_ncb(const T* L, const T* R, T* C, int64_t ld, int64_t m, int b, int skip, int slots,
                             hipStream_t st, hipEvent_t done) {
  if constexpr (KIND == KIND_LU) {
    constexpr int COLS = NCB * 16;
    const int npanels = (int)((m + kUpdRows - 1) / kUpdRows);
    const int nblk = (int)((m + COLS - 1) / COLS);
    const int c = npanels <= slots ? slots / npanels : 0;  // items per panel of the single launch
    // (large updates only: the second launch costs a launch gap and a left-panel load per short work item)
    if (m >= 4096 && c >= 1 && (int64_t)(c + 1) * 4 <= nblk && (int64_t)c * npanels * 10 < (int64_t)slots * 9) {
      const int first = slots / (c + 1);                     // panels of the first launch
      const int64_t rows_a = (int64_t)first * kUpdRows;
      if (first >= 1 && rows_a < m && skip <= rows_a) {
        int rc = launch_update_rows<T, KIND, NCB, KMAX>(L, R, C, ld, rows_a, m, b, skip, slots, st, nullptr);
        if (rc != DLA_SUCCESS) return rc;
        // at least four column blocks per work item in the second launch
        const int64_t rest_blocks = (int64_t)(npanels - first) * nblk;
        const int slots_b = rest_blocks / 4 < slots ? (int)(rest_blocks / 4) : slots;
        return launch_update_rows<T, KIND, NCB, KMAX>(L + rows_a * ld, R, C + rows_a * ld, ld, m - rows_a, m, b, 0, slots_b,
                                                      st, done);
      }
    }
  }
  return launch_update_rows<T, KIND, NCB, KMAX>(L, R, C, ld, m, m, b, skip, slots, st, done);
}

// fp32: 64-column blocks once every slot gets at least kWideMinBlocks of them (3-6 % faster at
// N = 8192), 32-column blocks below.  fp64 always takes 32-column blocks: three accumulator sets of
// a 64-column block do not fit the register file next to the left panel (it spills and halves the rate).
template <typename T, int KIND>
static int launch_update(const T* L, const T* R, T* C, int64_t ld, int64_t m, int b, int skip, int slots,
                         hipStream_t st, hipEvent_t done = nullptr) {
  if (m <= 0) return DLA_SUCCESS;
  // depth above 128 (two panels at once): the left panel takes twice the registers, the column blocks are 16 wide
  if (b > kUpdKMax) {
    // fp32 has the registers for 32-column blocks next to the deeper left panel (rows of C in 128-byte pieces, as
    // fp64; 64-column blocks were measured and are slower: LU 6.10 against 6.03 ms at N = 8192)
    if constexpr (sizeof(T) == 4) return launch_update_ncb<T, KIND, 2, 2 * kUpdKMax>(L, R, C, ld, m, b, skip, slots, st, done);
    else return launch_update_ncb<T, KIND, 1, 2 * kUpdKMax>(L, R, C, ld, m, b, skip, slots, st, done);
  }
  const int npanels = (int)((m + kUpdRows - 1) / kUpdRows);
  int64_t wide_blocks = 0;
  for (int p = 0; p < npanels; ++p) wide_blocks += update_blocks_of_panel(p, (int)m, KIND == KIND_CHOL, 64);
  if constexpr (sizeof(T) == 4) {  // the wide form does not fit the register file in fp64
    if (wide_blocks >= (int64_t)kWideMinBlocks * slots)
      return launch_update_ncb<T, KIND, 4>(L, R, C, ld, m, b, skip, slots, st, done);
  }
  return launch_update_ncb<T, KIND, 2>(L, R, C, ld, m, b, skip, slots, st, done);
}

template <typename T, int KIND>
static int launch_solve(SolveArgs<T> sa, hipStream_t st, hipEvent_t done = nullptr) {
  if (sa.b % kIb != 0) return DLA_ERR_UNSUPPORTED_PARAMS;  // a panel with something behind it is always nb wide
  auto kern = solve_kernel<T, KIND>;
  static LdsLimitOnce lds_limit;
  if (!lds_limit.ensure(reinterpret_cast<const void*>(kern), solve_lds_bytes<T>())) return DLA_ERR_HIP;
  const int per_wg = (kSolveThreads / 64) * kIb;  // panel rows/columns one workgroup solves
  const int wgs = (sa.m + per_wg - 1) / per_wg;
  sa.n_top = (KIND == KIND_LU) ? wgs : 0;
  const int grid = sa.n_top + wgs;
  if (grid <= 0) return DLA_SUCCESS;
  ProfileScope scope(PHASE_TRSM, 0.0, st);
  launch_ev(kern, dim3((unsigned)grid), dim3(kSolveThreads), solve_lds_bytes<T>(), st, done, sa);
  return launch_status(__func__);
}

template <typename T, int KIND>
static int launch_head(const HeadArgs<T>& a, hipStream_t st, hipEvent_t done, int* workgroups) {
  auto kern = head_kernel<T, KIND>;
  constexpr int lds = head_lds_bytes<T, KIND>();
  static LdsLimitOnce lds_limit;
  if (!lds_limit.ensure(reinterpret_cast<const void*>(kern), lds)) return DLA_ERR_HIP;
  const int nt = (a.bn + kHeadTile - 1) / kHeadTile;
  const int grid = (KIND == KIND_LU) ? nt * nt : nt * (nt + 1) / 2;
  *workgroups = grid;
  ProfileScope scope(PHASE_TRSM, 0.0, st);
  launch_ev(kern, dim3((unsigned)grid), dim3(kHeadThreads), lds, st, done, a);
  return launch_status(__func__);
}

// Helper streams and events for look-ahead: library-owned, default priority, created on first use
// and kept for the life of the process.
struct LookaheadCtx {
  hipStream_t head = nullptr;   // head updates
  hipStream_t panel = nullptr;  // panel solves + strip updates
  hipStream_t bulk = nullptr;   // bulk trailing updates
  hipEvent_t ev[8] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
  double ticks_per_s = 1e8;     // rate of the constant wall clock the in-kernel waits are bounded by
  bool ok = false;
};
// data: a device pointer of the call (its device is made current for a host thread that has none yet).
static LookaheadCtx& lookahead_ctx(const void* data) {
  static LookaheadCtx ctx;
  if (!ctx.ok) {
    // A host thread that has made no runtime call of its own may have no current device (stream creation
    // then fails with hipErrorNoDevice): give it the device the caller's matrix lives on.
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess || cur < 0) {
      hipPointerAttribute_t attr;
      int dev = 0;
      if (hipPointerGetAttributes(&attr, data) == hipSuccess) dev = attr.device;
      (void)hipGetLastError();
      (void)hipSetDevice(dev);
    }
    auto make_stream = [](hipStream_t* s) {
      if (*s) return true;  // kept from an earlier, incomplete attempt
      hipError_t e = hipStreamCreateWithFlags(s, hipStreamNonBlocking);
      if (e == hipErrorNoDevice) {  // (seen on worker threads of a host program that set the device elsewhere)
        (void)hipGetLastError();
        (void)hipSetDevice(0);
        e = hipStreamCreateWithFlags(s, hipStreamNonBlocking);
      }
      return hip_note(e, "hipStreamCreateWithFlags") == 0;
    };
    bool good = make_stream(&ctx.head) && make_stream(&ctx.panel) && make_stream(&ctx.bulk);
    for (int i = 0; i < 8 && good; ++i)
      if (!ctx.ev[i]) good = hip_note(hipEventCreateWithFlags(&ctx.ev[i], hipEventDisableTiming), "hipEventCreateWithFlags") == 0;
    int dev = 0, khz = 0;
    if (good && hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) == hipSuccess && khz > 0)
      ctx.ticks_per_s = 1e3 * (double)khz;
    ctx.ok = good;
  }
  return ctx;
}

// Schedule of the small strip updates (skinny products with k = nb): small tiles, so a panel
// that is only a few hundred rows long still spreads over many compute units, and the whole k
// extent in one slab, so a tile costs one round of global loads instead of one per slab (these
// launches sit on the latency chain and run beside a bulk update that keeps the memory busy).
// That variant needs a compute unit's registers to itself, so it is used once the bulk update has
// become small (late steps); beside a large bulk update the 16-deep slabs share compute units better.
// The strips of the fp64 LU beside a large bulk update are bound by the matrix pipes of the few compute
// units they get: there 64 x 64 tiles, which do twice the work per LDS byte of 32 x 32 ones, take over earlier
// (measured with the reserve of 64 units: LU N = 4000 1.99 -> 1.95 ms; fp32 LU and fp64 Cholesky lose 3 % at
// N = 8192 with them).
template <typename T, int KIND>
static GemmSchedule panel_schedule(int64_t mr) {
  if constexpr (sizeof(T) == 8 && KIND == KIND_LU) return mr <= 1536 ? GemmSchedule{32, 32, 128, 8, 16, 16} : GemmSchedule{64, 64, 16, 4, 32, 32};
  return mr <= 2304 ? GemmSchedule{32, 32, 128, 8, 16, 16} : GemmSchedule{32, 32, 16, 4, 16, 16};
}

template <typename T, int KIND>
static int factor_impl(T* A, int64_t n, int64_t lda, const dla_factor_params* p, void* ws, size_t ws_bytes,
                       hipStream_t st, int* d_info) {
  const dla_dtype dt = sizeof(T) == 8 ? DLA_F64 : DLA_F32;
  FactorPlan plan;
  GemmSchedule upd;
  const int op = (KIND == KIND_LU) ? OP_SUB : OP_SUB_NT_LOWER;
  int rc = resolve_factor_params(dt, n, p, op, &plan, &upd);
  if (rc != DLA_SUCCESS) return rc;
  const int nb = plan.nb, lookahead = plan.lookahead;  // nb: the sub-panel one diagonal-block kernel factors
  if (n == 0) return DLA_SUCCESS;
  if (!ws || ws_bytes < factor_workspace_bytes_impl(n, dt, p) || ((uintptr_t)ws % 256)) return DLA_ERR_WORKSPACE;
  // the panel-stationary update kernel unless the caller names any field of a tiled schedule
  const bool auto_tile = !(p && (p->update.tile_m != 0 || p->update.tile_n != 0 || p->update.tile_k != 0 ||
                                 p->update.unroll_k != 0 || p->update.wave_m != 0 || p->update.wave_n != 0));

  unsigned char* wsb = static_cast<unsigned char*>(ws);
  const size_t set = inv_set_bytes(dt);
  auto inv_lo_of = [&](int step) { return reinterpret_cast<T*>(wsb + (size_t)(2 * (step & 1)) * set); };
  auto inv_up_of = [&](int step) { return reinterpret_cast<T*>(wsb + (size_t)(2 * (step & 1) + 1) * set); };

  auto head_top_of = [&](int step) { return reinterpret_cast<T*>(wsb + 4 * set + (size_t)(2 * (step & 1)) * head_copy_bytes(dt)); };
  auto head_side_of = [&](int step) {
    return reinterpret_cast<T*>(wsb + 4 * set + (size_t)(2 * (step & 1) + 1) * head_copy_bytes(dt));
  };

  // hand-over counters of the look-ahead chain: [0] diagonal blocks factored, [1] head workgroups
  // finished, [2] set when a wait gave up
  int* const chain = reinterpret_cast<int*>(wsb + 4 * set + 4 * head_copy_bytes(dt));
  bool chained = false;  // set by the look-ahead path
  int heads_done = 0;    // head workgroups launched so far = what the next diagonal block waits for
  // A kernel of the chain may sit behind the largest bulk update of the call: its wait lasts at most a
  // tenth of a second plus eight times that update's duration at a tenth of the matrix-pipe peak.
  long long wait_ticks = 0;  // set with the pipeline's context
  auto diag = [&](int64_t k0, int step, hipStream_t s, hipEvent_t done) -> int {
    DiagArgs<T> da;
    da.A = A + k0 * lda + k0;
    da.lda = lda;
    da.b = (int)((n - k0 < nb) ? n - k0 : nb);
    da.k0 = (int)k0;
    da.info = d_info;
    da.inv_lo = inv_lo_of(step);
    da.inv_up = inv_up_of(step);
    da.wait_counter = chained ? chain + 1 : nullptr;  // head workgroups finished so far
    da.wait_target = heads_done;
    da.done_counter = chained ? chain : nullptr;
    da.broken = chained ? chain + 2 : nullptr;
    da.wait_ticks = wait_ticks;
    return launch_diag<T, KIND>(da, s, done);
  };
  // panel solves of the block column / block row behind diagonal block k0
  auto solves = [&](int64_t k0, int step, hipStream_t s, hipEvent_t done) -> int {
    const int b = (int)((n - k0 < nb) ? n - k0 : nb);
    const int64_t m = n - k0 - b;
    if (m == 0) return DLA_SUCCESS;
    T* const Akk = A + k0 * lda + k0;
    SolveArgs<T> sa;
    sa.D = Akk;
    sa.top = Akk + b;                  // A12: b x m
    sa.side = Akk + (int64_t)b * lda;  // A21: m x b
    sa.lda = lda;
    sa.b = b;
    sa.m = (int)m;
    sa.n_top = 0;
    sa.inv_lo = inv_lo_of(step);
    sa.inv_up = inv_up_of(step);
    return launch_solve<T, KIND>(sa, s, done);
  };
  // trailing-update schedule for an m x m update when the caller names the tile
  auto update_schedule = [&](int64_t) { return upd; };

  // mm x mm trailing update behind the panel whose L21 / U12 are given.  skip > 0: the leading
  // skip x skip block of the region is left alone (another stream owns it).
  // In the look-ahead pipeline the bulk update leaves a few compute units free: its workgroups fill
  // a compute unit's registers, so the small kernels of the latency chain (diagonal block, head
  // update) would otherwise queue behind a whole bulk update.
  const bool pipelined = lookahead && n > 2 * (int64_t)nb;
  // Cholesky's zero upper triangle can be written early when nothing dirties it later: the default update
  // kernel works on 128-row panels and stays inside the 128-wide block diagonal; other block sizes or a tiled
  // update write above it, and the triangle is zeroed at the end instead.
  const bool early_zero = KIND == KIND_CHOL && pipelined && nb == kUpdRows && auto_tile;
  const int slots = pipelined ? kNumCu - kChainCu : kNumCu;
  const int slots_wide = pipelined ? kNumCu - (sizeof(T) == 8 ? kChainCuWide : kChainCu) : kNumCu;
  auto trailing_gemm = [&](const T* Lp, const T* Up, T* Cp, int64_t mm, int bb, int skip, hipStream_t s) -> int {
    const GemmSchedule us = update_schedule(mm);
    if (skip == 0) {
      if (KIND == KIND_LU) return run_gemm<T>(us, OP_SUB, Lp, lda, Up, lda, Cp, lda, mm, mm, bb, s);
      return run_gemm<T>(us, OP_SUB_NT_LOWER, Lp, lda, Lp, lda, Cp, lda, mm, mm, bb, s);
    }
    // region minus its leading block: the rows below the block over the full width, and (LU) the
    // block's rows to the right of it
    const int64_t rest = mm - skip;
    if (rest <= 0) return DLA_SUCCESS;
    int r;
    if (KIND == KIND_LU) {
      if ((r = run_gemm<T>(us, OP_SUB, Lp, lda, Up + skip, lda, Cp + skip, lda, skip, rest, bb, s)) != DLA_SUCCESS) return r;
      return run_gemm<T>(us, OP_SUB, Lp + (int64_t)skip * lda, lda, Up, lda, Cp + (int64_t)skip * lda, lda, rest, mm, bb, s);
    }
    const T* Lr = Lp + (int64_t)skip * lda;
    if ((r = run_gemm<T>(us, OP_SUB_NT, Lr, lda, Lp, lda, Cp + (int64_t)skip * lda, lda, rest, skip, bb, s)) != DLA_SUCCESS)
      return r;
    return run_gemm<T>(us, OP_SUB_NT_LOWER, Lr, lda, Lr, lda, Cp + (int64_t)skip * lda + skip, lda, rest, rest, bb, s);
  };
  // done (optional): event that completes with the update
  auto trailing = [&](const T* Lp, const T* Up, T* Cp, int64_t mm, int bb, int skip, hipStream_t s,
                      hipEvent_t done) -> int {
    if (auto_tile)
      return launch_update<T, KIND>(Lp, KIND == KIND_LU ? Up : Lp, Cp, lda, mm, bb, skip, (mm >= kWideReserveMinRows && mm < kWideReserveMaxRows) ? slots_wide : slots,
                                    s, done);
    const int r = trailing_gemm(Lp, Up, Cp, mm, bb, skip, s);
    if (r != DLA_SUCCESS) return r;
    if (done && hip_note(hipEventRecord(done, s), "hipEventRecord") != 0) return DLA_ERR_HIP;
    return DLA_SUCCESS;
  };

  if (!pipelined) {
    // one stream, strictly sequential steps
    int step = 0;
    for (int64_t k0 = 0; k0 < n; k0 += nb, ++step) {
      const int b = (int)((n - k0 < nb) ? n - k0 : nb);
      const int64_t m = n - k0 - b;
      if ((rc = diag(k0, step, st, nullptr)) != DLA_SUCCESS) return rc;
      if (m == 0) break;
      if ((rc = solves(k0, step, st, nullptr)) != DLA_SUCCESS) return rc;
      T* const Akk = A + k0 * lda + k0;
      if ((rc = trailing(Akk + (int64_t)b * lda, Akk + b, Akk + (int64_t)b * lda + b, m, b, 0, st, nullptr)) != DLA_SUCCESS) return rc;
    }
  } else {
    // Look-ahead pipeline over four streams.  With N = block k+1 and N2 = block k+2:
    //   caller's stream   diag(k): factor diagonal block k                 } the latency chain,
    //   head stream       head(k): block (N,N) gets step k's update from   } nothing else on
    //                     the un-solved panel heads                        } these two streams
    //   panel stream      solves(k): the full panel solves;  strips(k): step k's update of block
    //                     row N and block column N (what solves(k+1) reads) and of block (N2,N2)
    //                     (what head(k+1) reads)
    //   bulk stream       bulk(k): step k's update of everything behind block row/column N except
    //                     block (N2,N2)
    // Dependencies: head(k) after diag(k) and strips(k-1); diag(k+1) after head(k); solves(k) after
    // diag(k); strips(k) after bulk(k-1) (same memory); bulk(k) after solves(k).  Host order of a
    // step: head(k), diag(k+1), solves(k), strips(k), bulk(k).
    // solves(k) overwrites the panel heads A[k][N], A[N][k] that head(k) reads, so strips(k-1), which
    // produces those two blocks, also writes a copy of them to the workspace and head(k) reads the
    // copies; only the first step reads them in place and makes solves(0) wait for head(0).
    //
    // The chain diag(k) -> head(k) -> diag(k+1) alternates between the caller's stream and the head
    // stream, and each of its kernels is launched while its predecessor still runs: it waits for it
    // on a counter in the workspace instead of a stream dependency, which hides its launch latency.
    // Every kernel is submitted after everything it waits for, so the order of submission is a valid
    // order of execution whatever hardware queues the streams share.  It does need kernels of this
    // process to run side by side; where they cannot (a profiler collecting hardware counters
    // serialises them), lookahead = 2 keeps the same streams and orders the chain with events.
    //
    // Only the chain is handed over this way: a waiting kernel holds its compute units, and the
    // bulk update needs every unit outside the reserve at once, so a head update that also waited
    // in place for the strips (tried) doubled the bulk update's run time.
    // The helper streams and events are shared by every call of the process: one call enqueues its
    // whole pipeline before the next one starts to, so calls from several host threads line up on
    // the helper streams instead of mixing their events.
    static std::mutex submit_mutex;
    std::lock_guard<std::mutex> submit_lock(submit_mutex);
    LookaheadCtx& ctx = lookahead_ctx(A);
    if (!ctx.ok) return DLA_ERR_HIP;  // (the failing call is on record)
    wait_ticks = (long long)(ctx.ticks_per_s * (0.1 + 8.0 * (2.0 * (double)n * (double)n * 2.0 * nb) / 8e12));
    hipEvent_t e_head = ctx.ev[0], e_solve = ctx.ev[1], e_bulk = ctx.ev[2], e_start = ctx.ev[3], e_strip = ctx.ev[6];
    hipEvent_t e_diag[2] = {ctx.ev[4], ctx.ev[5]};  // by step parity
    constexpr int SOP = (KIND == KIND_LU) ? OP_SUB : OP_SUB_NT;
    const int nsteps = (int)((n + nb - 1) / nb) - 1;  // steps that have a panel behind the diagonal block
    bool bulk_pending = false;
    // Two-level blocking of the bulk update while the trailing matrix is large (the bulk stream is then the
    // longest): every other step puts its bulk update off (owed), and the step after it carries both
    // panels as one update of depth 2 nb, which halves the traffic of the trailing matrix per flop.  So
    // that nothing on the side path has to wait for that longer update, the strips of such a wide step
    // also take block row / column N2 and block (N3,N3), and its bulk update starts behind them; the
    // next step's strips then touch nothing the bulk update writes (after_wide).
    bool owed = false, after_wide = false;

    // ---- panel and bulk streams of one step
    auto panel_side = [&](int step) -> int {
      const int64_t k0 = (int64_t)step * nb;
      const int b = nb;  // only the last diagonal block can be short, and it has no panel
      const int64_t m = n - k0 - b;
      T* const Akk = A + k0 * lda + k0;
      T* const L21 = Akk + (int64_t)b * lda;  // m x b
      T* const U12 = Akk + b;                 // b x m   (LU)
      T* const A22 = L21 + b;
      const int64_t bn = m < nb ? m : nb;     // size of block N
      const int64_t mr = m - bn;              // what is left behind it
      const int64_t bn2 = mr < nb ? mr : nb;  // size of block N2
      const bool wide = owed;                 // this step also applies the previous step's panels
      const int ksh = wide ? nb : 0;          // depth added in front of this step's panels
      const int kk = b + ksh;
      const int64_t lsh = ksh, ush = (KIND == KIND_LU) ? (int64_t)ksh * lda : (int64_t)ksh;
      int r;
      // solves(k) behind diag(k).  With the chain's counters in use that is a one-wave kernel in front of the solves
      // that waits in place for the count of factored blocks: on the host a plain launch costs a quarter of a wait
      // for another stream's event (2.6 against 10 us), and the host's submission time per step is as long as the
      // step; on the device the solves start a same-stream launch gap after the block is done instead of an event's
      // round trip.  (Submitted after diag(k), like everything that waits for it.)
      if (chained && step > 0) {
        hipLaunchKernelGGL(gate_kernel, dim3(1), dim3(64), 0, ctx.panel, (const int*)chain, step + 1, chain + 2, wait_ticks);
        if (launch_status(__func__) != DLA_SUCCESS) return DLA_ERR_HIP;
      } else if (hip_note(hipStreamWaitEvent(ctx.panel, step == 0 ? e_head : e_diag[step & 1], 0), "hipStreamWaitEvent") != 0) {
        return DLA_ERR_HIP;
      }
      // the last kernel of the step on this stream carries e_strip
      if ((r = solves(k0, step, ctx.panel, mr > 0 ? e_solve : e_strip)) != DLA_SUCCESS) return r;
      if (mr > 0) {
        if (bulk_pending && !after_wide && hip_note(hipStreamWaitEvent(ctx.panel, e_bulk, 0), "hipStreamWaitEvent") != 0) return DLA_ERR_HIP;
        const T* Lr = L21 + bn * lda;  // rows behind block N of the solved column panel
        const GemmSchedule ps = panel_schedule<T, KIND>(mr);
        GemmGroup<T> g;
        int np = 0, tiles = 0;
        double flops = 0.0;
        auto add = [&](const T* a, const T* bm, T* c, int64_t M, int64_t N, T* copy) {
          if (M <= 0 || N <= 0) return;
          g.prob[np] = make_problem<T>(ps, SOP, a - lsh, lda, bm - ush, lda, c, lda, M, N, kk, tiles);
          g.prob[np].C2 = copy;
          g.prob[np].ldc2 = kNbMax;
          tiles += problem_tiles(ps, SOP, g.prob[np]);
          flops += 2.0 * (double)M * (double)N * (double)kk;
          ++np;
        };
        const int64_t rest = mr - bn2;  // rows / columns behind block N2
        T* const side_copy = head_side_of(step + 1);  // A[N2][N], the next step's column-panel head
        T* const top_copy = head_top_of(step + 1);    // A[N][N2], the next step's row-panel head
        if (KIND == KIND_LU) {
          add(Lr, U12, A22 + bn * lda, bn2, bn, side_copy);                              // block (N2,N)
          add(Lr + bn2 * lda, U12, A22 + (bn + bn2) * lda, rest, bn, nullptr);           // block column N below it
          add(L21, U12 + bn, A22 + bn, bn, bn2, top_copy);                               // block (N,N2)
          add(L21, U12 + bn + bn2, A22 + bn + bn2, bn, rest, nullptr);                   // block row N right of it
          add(Lr, U12 + bn, A22 + bn * lda + bn, bn2, bn2, nullptr);                     // block (N2,N2)
        } else {
          add(Lr, L21, A22 + bn * lda, bn2, bn, side_copy);                              // block (N2,N)
          add(Lr + bn2 * lda, L21, A22 + (bn + bn2) * lda, rest, bn, nullptr);           // block column N below it
          add(Lr, Lr, A22 + bn * lda + bn, bn2, bn2, nullptr);                           // block (N2,N2)
        }
        auto launch_group = [&](hipEvent_t done) -> int {
          if (np == 0) return DLA_SUCCESS;
          for (int q = np; q < kMaxGroup; ++q) g.prob[q] = g.prob[0];
          g.nprob = np;
          g.total_tiles = tiles;
          ProfileScope scope(PHASE_GEMM, flops, ctx.panel);
          tl_gemm_done_event = done;
          const int rr = launch_gemm<T>(ps, SOP, g, ctx.panel);
          np = tiles = 0;
          flops = 0.0;
          return rr;
        };
        if ((r = launch_group(e_strip)) != DLA_SUCCESS) return r;
        if (wide) {
          // block row / column N2 behind block (N2,N2), and block (N3,N3): what the next step's strips work on
          const int64_t bn3 = rest < nb ? rest : nb, o2 = bn + bn2;
          const T* Lr3 = Lr + bn2 * lda;  // rows from block N3 on
          if (KIND == KIND_LU) {
            add(Lr3, U12 + bn, A22 + o2 * lda + bn, rest, bn2, nullptr);       // block column N2 below (N2,N2)
            add(Lr, U12 + o2, A22 + bn * lda + o2, bn2, rest, nullptr);         // block row N2 right of it
            add(Lr3, U12 + o2, A22 + o2 * lda + o2, bn3, bn3, nullptr);         // block (N3,N3)
          } else {
            add(Lr3, Lr, A22 + o2 * lda + bn, rest, bn2, nullptr);              // block column N2 below (N2,N2)
            add(Lr3, Lr3, A22 + o2 * lda + o2, bn3, bn3, nullptr);              // block (N3,N3)
          }
          if ((r = launch_group(nullptr)) != DLA_SUCCESS) return r;
        }
      }
      if (mr > bn2) {
        const int64_t rest = mr - bn2;
        // put the bulk update off when the step after this one can carry it: full blocks N2, N3 and
        // two more behind them, and a trailing matrix large enough for the bulk stream to be the longest
        if (!owed && auto_tile && plan.two_level && mr >= plan.defer_min_rows && rest >= 4 * (int64_t)nb) {
          owed = true;
          after_wide = false;
          return DLA_SUCCESS;
        }
        if (hip_note(hipStreamWaitEvent(ctx.bulk, e_solve, 0), "hipStreamWaitEvent") != 0) return DLA_ERR_HIP;
        if (wide) {
          const int64_t bn3 = rest < nb ? rest : nb, o2 = bn + bn2;
          if ((r = trailing(L21 + o2 * lda - lsh, U12 + o2 - ush, A22 + o2 * lda + o2, rest, kk, (int)bn3, ctx.bulk, e_bulk)) !=
              DLA_SUCCESS)
            return r;
        } else if ((r = trailing(L21 + bn * lda, U12 + bn, A22 + bn * lda + bn, mr, b, (int)bn2, ctx.bulk, e_bulk)) != DLA_SUCCESS) {
          return r;
        }
        bulk_pending = true;
      }
      owed = false;
      after_wide = wide;
      return DLA_SUCCESS;
    };

    // ---- the chain of one step: head(k), diag(k+1)
    auto chain_side = [&](int step) -> int {
      const int64_t k0 = (int64_t)step * nb;
      const int b = nb;
      const int64_t m = n - k0 - b;
      T* const Akk = A + k0 * lda + k0;
      const int64_t bn = m < nb ? m : nb;
      if (step > 0 && hip_note(hipStreamWaitEvent(ctx.head, e_strip, 0), "hipStreamWaitEvent") != 0) return DLA_ERR_HIP;
      if (!chained && hip_note(hipStreamWaitEvent(ctx.head, e_diag[step & 1], 0), "hipStreamWaitEvent") != 0) return DLA_ERR_HIP;
      HeadArgs<T> ha;
      ha.D = Akk;
      ha.top = step == 0 ? Akk + b : head_top_of(step);
      ha.side = step == 0 ? Akk + (int64_t)b * lda : head_side_of(step);
      ha.C = Akk + (int64_t)b * lda + b;
      ha.lda = lda;
      ha.ldh = step == 0 ? lda : kNbMax;
      ha.b = b;
      ha.bn = (int)bn;
      ha.inv_lo = inv_lo_of(step);
      ha.inv_up = inv_up_of(step);
      ha.wait_counter = chained ? chain : nullptr;  // diagonal blocks factored: block k is number k + 1
      ha.wait_target = step + 1;
      ha.done_counter = chained ? chain + 1 : nullptr;
      ha.broken = chain + 2;
      ha.wait_ticks = wait_ticks;
      int head_wgs = 0, r;
      if ((r = launch_head<T, KIND>(ha, ctx.head, e_head, &head_wgs)) != DLA_SUCCESS) return r;
      heads_done += head_wgs;
      if (!chained && hip_note(hipStreamWaitEvent(st, e_head, 0), "hipStreamWaitEvent") != 0) return DLA_ERR_HIP;
      if ((r = diag(k0 + b, step + 1, st, chained ? nullptr : e_diag[(step + 1) & 1])) != DLA_SUCCESS) return r;
      return DLA_SUCCESS;
    };

    // a wait that gives up can only be reported through d_info: without it the chain is ordered by events
    chained = lookahead == 1 && d_info != nullptr;
    // A call starts behind the previous pipelined call of the process: its first kernels would
    // otherwise wait in place for work that is queued behind that call on the helper streams.
    hipEvent_t e_call_done = ctx.ev[7];
    if (hip_note(hipStreamWaitEvent(st, e_call_done, 0), "hipStreamWaitEvent") != 0) return DLA_ERR_HIP;
    hipLaunchKernelGGL(zero_ints_kernel, dim3(1), dim3(64), 0, st, chain, 3);
    if (launch_status(__func__) != DLA_SUCCESS) return DLA_ERR_HIP;
    if (hipEventRecord(e_start, st) != hipSuccess || hipStreamWaitEvent(ctx.head, e_start, 0) != hipSuccess)
      return DLA_ERR_HIP;
    if ((rc = diag(0, 0, st, chained ? nullptr : e_diag[0])) != DLA_SUCCESS) return rc;
    if (early_zero) {
      // the output's zero upper triangle: the blocks above the block diagonal now, on the panel stream, beside
      // the first steps (nothing reads or writes them); each diagonal block's own upper part by its kernel
      if (hip_note(hipStreamWaitEvent(ctx.panel, e_start, 0), "hipStreamWaitEvent") != 0) return DLA_ERR_HIP;
      hipLaunchKernelGGL(zero_upper_kernel<T>, dim3((unsigned)((n + 255) / 256), (unsigned)(n < 32768 ? n : 32768)),
                         dim3(256), 0, ctx.panel, A, lda, (int)n, nb);
      if (launch_status(__func__) != DLA_SUCCESS) return DLA_ERR_HIP;
    }

    for (int step = 0; step < nsteps; ++step) {
      if ((rc = chain_side(step)) != DLA_SUCCESS) return rc;
      if ((rc = panel_side(step)) != DLA_SUCCESS) return rc;
    }
    // join: everything the helper streams did becomes part of the caller's stream
    if (hip_note(hipStreamWaitEvent(st, e_head, 0), "hipStreamWaitEvent") != 0) return DLA_ERR_HIP;
    if (hip_note(hipStreamWaitEvent(st, e_strip, 0), "hipStreamWaitEvent") != 0) return DLA_ERR_HIP;
    if (bulk_pending && hip_note(hipStreamWaitEvent(st, e_bulk, 0), "hipStreamWaitEvent") != 0) return DLA_ERR_HIP;
    if (hip_note(hipEventRecord(e_call_done, st), "hipEventRecord") != 0) return DLA_ERR_HIP;
  }
  if (KIND == KIND_CHOL && n > 1 && !early_zero) {
    hipLaunchKernelGGL(zero_upper_kernel<T>, dim3((unsigned)((n + 255) / 256), (unsigned)(n < 32768 ? n : 32768)),
                       dim3(256), 0, st, A, lda, (int)n, 1);
    if (launch_status(__func__) != DLA_SUCCESS) return DLA_ERR_HIP;
  }
  return DLA_SUCCESS;
}

template <typename T>
int rank_update_impl(bool lower, const T* L, const T* Rm, T* C, int64_t ld, int64_t m, int b, hipStream_t st) {
  if (lower) return launch_update<T, KIND_CHOL>(L, L, C, ld, m, b, 0, kNumCu, st);
  return launch_update<T, KIND_LU>(L, Rm, C, ld, m, b, 0, kNumCu, st);
}
template int rank_update_impl<double>(bool, const double*, const double*, double*, int64_t, int64_t, int, hipStream_t);
template int rank_update_impl<float>(bool, const float*, const float*, float*, int64_t, int64_t, int, hipStream_t);

// Diagnostic: one diagonal-block kernel told to wait for a predecessor that does not exist.  It
// must give up after the bounded poll, mark the pipeline broken and report -1, and exit normally.
// scratch: >= kHandoverSelftestBytes, 256-byte aligned: a 16 x 16 identity, its inverses, counters.
int handover_selftest_impl(void* scratch, hipStream_t st, int* d_info) {
  double* const A = static_cast<double*>(scratch);  // 16 x 16
  double* const inv = A + 256;                      // 2 x 256
  int* const chain = reinterpret_cast<int*>(inv + 512);
  hipLaunchKernelGGL(identity16_kernel, dim3(1), dim3(256), 0, st, A, chain);
  if (launch_status(__func__) != DLA_SUCCESS) return DLA_ERR_HIP;
  DiagArgs<double> da;
  da.A = A;
  da.lda = 16;
  da.b = 16;
  da.k0 = 16;  // not the first block of a call: info is only touched to report
  da.info = d_info;
  da.inv_lo = inv;
  da.inv_up = inv + 256;
  da.wait_counter = chain + 1;
  da.wait_target = 1;  // nobody will ever count to one
  da.done_counter = chain;
  da.broken = chain + 2;
  da.wait_ticks = 5000000;  // 0.05 s at the usual 100 MHz
  return launch_diag<double, KIND_LU>(da, st, nullptr);
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
