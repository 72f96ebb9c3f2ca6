// C-ABI entry points (see include/dla.h): argument validation, schedule
// resolution, 3mm driver, GEMM export, profiler.  Argument errors are reported
// before any HIP call so they can be exercised on a machine without a GPU.
#include <cstdio>
#include <mutex>
#include <vector>
#include "host_common.hpp"

namespace dla {

// ------------------------------------------------------------------ schedule menu
struct TileEntry {
  int tm, tn, wm, wn;
};
static const TileEntry kTiles[] = {
#define DLA_ROW(TM, TN, WM, WN) {TM, TN, WM, WN},
    DLA_TILE_MENU(DLA_ROW)
#undef DLA_ROW
};
struct KuEntry {
  int tk, uk;
};
static const KuEntry kKu[] = {
#define DLA_ROW(TK, UK) {TK, UK},
    DLA_KU_MENU(DLA_ROW)
#undef DLA_ROW
};
static const int kNumTiles = (int)(sizeof(kTiles) / sizeof(kTiles[0]));
static const int kNumKu = (int)(sizeof(kKu) / sizeof(kKu[0]));

static int esize(dla_dtype dt) { return dt == DLA_F64 ? 8 : 4; }

int resolve_schedule(dla_dtype dt, const dla_gemm_params* in, int op, GemmSchedule* out, int64_t m, int64_t n) {
  GemmSchedule s = {0, 0, 0, 0, 0, 0};
  if (in) s = GemmSchedule{in->tile_m, in->tile_n, in->tile_k, in->unroll_k, in->wave_m, in->wave_n};
  if (s.tm < 0 || s.tn < 0 || s.tk < 0 || s.uk < 0 || s.wm < 0 || s.wn < 0) return DLA_ERR_UNSUPPORTED_PARAMS;
  if (s.tm == 0 && s.tn == 0) {
    // A 128x128 macro-tile needs about four tiles per compute unit to balance the 256 of them;
    // outputs smaller than that (the 3mm products of the paper's datasets) take 64x64 tiles.
    const bool small = m > 0 && n > 0 && ((m + 127) / 128) * ((n + 127) / 128) < 4 * 256;
    s.tm = s.tn = small ? 64 : 128;
    if (small && s.tk == 0 && s.uk == 0) {
      s.tk = 16;
      s.uk = 4;  // the whole 16-deep slab unrolled: 4-8 % faster than 2 on the 3mm products
    }
  }
  if (s.tm == 0) s.tm = s.tn;
  if (s.tn == 0) s.tn = s.tm;
  if (s.wm == 0 || s.wn == 0) {  // default wave split: first menu row with this macro-tile
    bool found = false;
    for (int i = 0; i < kNumTiles && !found; ++i)
      if (kTiles[i].tm == s.tm && kTiles[i].tn == s.tn && (s.wm == 0 || s.wm == kTiles[i].wm) &&
          (s.wn == 0 || s.wn == kTiles[i].wn)) {
        s.wm = kTiles[i].wm;
        s.wn = kTiles[i].wn;
        found = true;
      }
    if (!found) return DLA_ERR_UNSUPPORTED_PARAMS;
  }
  if (s.tk == 0) s.tk = 16;
  if (s.uk == 0) {  // largest unroll instantiated for this slab depth
    for (int i = 0; i < kNumKu; ++i)
      if (kKu[i].tk == s.tk && kKu[i].uk > s.uk) s.uk = kKu[i].uk;
    if (s.uk == 0) return DLA_ERR_UNSUPPORTED_PARAMS;
  }
  bool tile_ok = false, ku_ok = false;
  for (int i = 0; i < kNumTiles; ++i)
    tile_ok |= (kTiles[i].tm == s.tm && kTiles[i].tn == s.tn && kTiles[i].wm == s.wm && kTiles[i].wn == s.wn);
  for (int i = 0; i < kNumKu; ++i) ku_ok |= (kKu[i].tk == s.tk && kKu[i].uk == s.uk);
  if (!tile_ok || !ku_ok) return DLA_ERR_UNSUPPORTED_PARAMS;
  if (op == OP_SUB_NT_LOWER && s.tm != s.tn) return DLA_ERR_UNSUPPORTED_PARAMS;
  if (gemm_lds_bytes(s, op == OP_SUB_NT_LOWER || op == OP_SUB_NT, esize(dt)) > kMaxLdsBytes)
    return DLA_ERR_UNSUPPORTED_PARAMS;
  *out = s;
  return DLA_SUCCESS;
}

// ------------------------------------------------------------------ profiler
struct ProfileRecord {
  hipEvent_t e0, e1;
  int phase;
  double flops;
};
static bool g_profile_on = false;
static std::vector<ProfileRecord> g_records;
static std::vector<hipEvent_t> g_event_pool;
static std::mutex g_profile_mutex;

static hipEvent_t take_event() {
  if (!g_event_pool.empty()) {
    hipEvent_t e = g_event_pool.back();
    g_event_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

int profile_begin(int phase, double flops, hipStream_t st) {
  if (!g_profile_on) return -1;
  std::lock_guard<std::mutex> lock(g_profile_mutex);
  ProfileRecord r;
  r.e0 = take_event();
  r.e1 = take_event();
  r.phase = phase;
  r.flops = flops;
  if (!r.e0 || !r.e1) return -1;
  (void)hipEventRecord(r.e0, st);
  g_records.push_back(r);
  return (int)g_records.size() - 1;
}

bool profile_kernel_events(int phase, double flops, hipEvent_t* start, hipEvent_t* stop) {
  if (!g_profile_on) return false;
  std::lock_guard<std::mutex> lock(g_profile_mutex);
  ProfileRecord r;
  r.e0 = take_event();
  r.e1 = take_event();
  r.phase = phase;
  r.flops = flops;
  if (!r.e0 || !r.e1) return false;
  g_records.push_back(r);
  *start = r.e0;
  *stop = r.e1;
  return true;
}

void profile_end(int slot, hipStream_t st) {
  if (slot < 0) return;
  std::lock_guard<std::mutex> lock(g_profile_mutex);
  if (slot < (int)g_records.size()) (void)hipEventRecord(g_records[slot].e1, st);
}

// ------------------------------------------------------------------ GEMM wrapper
template <typename T>
int run_gemm(const GemmSchedule& s, int op, const T* A, int64_t lda, const T* B, int64_t ldb, T* C, int64_t ldc,
             int64_t M, int64_t N, int64_t K, hipStream_t st) {
  if (M <= 0 || N <= 0) return DLA_SUCCESS;
  GemmGroup<T> g;
  g.nprob = 1;
  g.prob[0] = make_problem<T>(s, op, A, lda, B, ldb, C, ldc, M, N, K, 0);
  for (int q = 1; q < kMaxGroup; ++q) g.prob[q] = g.prob[0];
  g.total_tiles = problem_tiles(s, op, g.prob[0]);
  const double flops = (op == OP_SUB_NT_LOWER ? 1.0 : 2.0) * (double)M * (double)N * (double)K;
  ProfileScope scope(PHASE_GEMM, flops, st);
  return launch_gemm<T>(s, op, g, st);
}
template int run_gemm<double>(const GemmSchedule&, int, const double*, int64_t, const double*, int64_t, double*,
                              int64_t, int64_t, int64_t, int64_t, hipStream_t);
template int run_gemm<float>(const GemmSchedule&, int, const float*, int64_t, const float*, int64_t, float*, int64_t,
                             int64_t, int64_t, int64_t, hipStream_t);

// C = 0 for the degenerate k == 0 product.
template <typename T>
__global__ void fill_zero_kernel(T* c, int64_t ld, int rows, int cols) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < (int64_t)rows * cols) c[(i / cols) * ld + (i % cols)] = T(0);
}
template <typename T>
static int fill_zero(T* c, int64_t ld, int64_t rows, int64_t cols, hipStream_t st) {
  if (rows <= 0 || cols <= 0) return DLA_SUCCESS;
  const int64_t total = rows * cols;
  hipLaunchKernelGGL(fill_zero_kernel<T>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, c, ld, (int)rows,
                     (int)cols);
  return launch_status(__func__);
}

static inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Mm3Layout {
  int64_t lde, ldf;
  size_t e_bytes, f_bytes;
};
static Mm3Layout mm3_layout(int64_t ni, int64_t nj, int64_t nl, dla_dtype dt) {
  Mm3Layout L;
  const size_t es = (size_t)esize(dt);
  L.lde = (int64_t)round_up((size_t)(nj > 0 ? nj : 1), 16);  // rows start on 64/128-byte boundaries
  L.ldf = (int64_t)round_up((size_t)(nl > 0 ? nl : 1), 16);
  L.e_bytes = round_up((size_t)(ni > 0 ? ni : 0) * (size_t)L.lde * es, 256);
  L.f_bytes = round_up((size_t)(nj > 0 ? nj : 0) * (size_t)L.ldf * es, 256);
  return L;
}

template <typename T>
static int mm3_impl(const T* A, int64_t lda, const T* B, int64_t ldb, const T* C, int64_t ldc, const T* D,
                    int64_t ldd, T* G, int64_t ldg, int64_t ni, int64_t nk, int64_t nj, int64_t nm, int64_t nl,
                    const GemmSchedule& se, const GemmSchedule& sf, const GemmSchedule& sg, void* ws,
                    hipStream_t st) {
  const Mm3Layout L = mm3_layout(ni, nj, nl, sizeof(T) == 8 ? DLA_F64 : DLA_F32);
  T* E = reinterpret_cast<T*>(ws);
  T* F = reinterpret_cast<T*>(reinterpret_cast<unsigned char*>(ws) + L.e_bytes);
  if (ni == 0 || nl == 0) return DLA_SUCCESS;  // G is empty
  int rc;
  if (nj == 0) return fill_zero(G, ldg, ni, nl, st);  // E and F are empty: G = 0
  // E = A*B and F = C*D are independent: one grouped launch when their schedules coincide.
  const bool same = se.tm == sf.tm && se.tn == sf.tn && se.tk == sf.tk && se.uk == sf.uk && se.wm == sf.wm &&
                    se.wn == sf.wn;
  if (nk == 0) { if ((rc = fill_zero(E, L.lde, ni, nj, st)) != DLA_SUCCESS) return rc; }
  if (nm == 0) { if ((rc = fill_zero(F, L.ldf, nj, nl, st)) != DLA_SUCCESS) return rc; }
  if (same && nk > 0 && nm > 0) {
    GemmGroup<T> g;
    g.nprob = 2;
    g.prob[0] = make_problem<T>(se, OP_ASSIGN, A, lda, B, ldb, E, L.lde, ni, nj, nk, 0);
    const int t0 = problem_tiles(se, OP_ASSIGN, g.prob[0]);
    g.prob[1] = make_problem<T>(se, OP_ASSIGN, C, ldc, D, ldd, F, L.ldf, nj, nl, nm, t0);
    g.total_tiles = t0 + problem_tiles(se, OP_ASSIGN, g.prob[1]);
    for (int q = 2; q < kMaxGroup; ++q) g.prob[q] = g.prob[1];
    ProfileScope scope(PHASE_GEMM, 2.0 * ((double)ni * nj * nk + (double)nj * nl * nm), st);
    if ((rc = launch_gemm<T>(se, OP_ASSIGN, g, st)) != DLA_SUCCESS) return rc;
  } else {
    if (nk > 0 && (rc = run_gemm<T>(se, OP_ASSIGN, A, lda, B, ldb, E, L.lde, ni, nj, nk, st)) != DLA_SUCCESS) return rc;
    if (nm > 0 && (rc = run_gemm<T>(sf, OP_ASSIGN, C, ldc, D, ldd, F, L.ldf, nj, nl, nm, st)) != DLA_SUCCESS) return rc;
  }
  return run_gemm<T>(sg, OP_ASSIGN, E, L.lde, F, L.ldf, G, ldg, ni, nl, nj, st);
}

static const int64_t kMaxDim = (int64_t)1 << 30;

// ------------------------------------------------------------------ scratch of mm3_noalloc
// E and F of a 3mm for callers that may not allocate: a fixed array in the device image, one copy per
// GPU, held from the moment the library's code is loaded on that GPU until the process ends.  In host
// code the array's name is only a handle for hipGetSymbolAddress; the device address it returns (one
// per GPU) is what is passed to kernels.
static __device__ __align__(256) unsigned char scratch[DLA_MM3_NOALLOC_MAX_BYTES];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (looked up once per device), or null on failure.
static void* scratch_of_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

// Register-resident MFMA loop: what the matrix pipes sustain when nothing else limits them.
template <typename T>
__global__ void __launch_bounds__(256) mfma_peak_kernel(T* out, int iters) {
  using acc_t = typename Mfma<T>::acc_t;
  constexpr int ILP = 4;
  acc_t acc[ILP];
#pragma unroll
  for (int i = 0; i < ILP; ++i) acc[i] = acc_t{0, 0, 0, 0};
  const T a = T(1e-3) * (T)threadIdx.x, b = T(1) + T(1e-4) * (T)threadIdx.x;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < ILP; ++i) acc[i] = Mfma<T>::mma(a, b, acc[i]);
  }
  T s = 0;
#pragma unroll
  for (int i = 0; i < ILP; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}
constexpr int kPeakGrid = 1024, kPeakIters = 4000;

template <typename T>
static int mfma_peak_impl(void* scratch, hipStream_t st, double* tflops) {
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return DLA_ERR_HIP;
  if (hipEventCreate(&e1) != hipSuccess) {
    (void)hipEventDestroy(e0);
    return DLA_ERR_HIP;
  }
  float best = 0.0f;
  bool ok = true;
  for (int rep = 0; rep < 3 && ok; ++rep) {  // first pass warms the clocks up, the fastest of three counts
    ok = hipEventRecord(e0, st) == hipSuccess;
    hipLaunchKernelGGL(mfma_peak_kernel<T>, dim3(kPeakGrid), dim3(256), 0, st, static_cast<T*>(scratch), kPeakIters);
    ok = ok && hipGetLastError() == hipSuccess && hipEventRecord(e1, st) == hipSuccess &&
         hipEventSynchronize(e1) == hipSuccess;
    float ms = 0.0f;
    ok = ok && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
    if (ok && ms > 0.0f && (best == 0.0f || ms < best)) best = ms;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (!ok || best <= 0.0f) return DLA_ERR_HIP;
  const double flops = (double)kPeakGrid * 4 /*waves*/ * kPeakIters * 4 /*ILP*/ * 2048.0;  // 16*16*4*2 per MFMA
  *tflops = flops / (best * 1e-3) * 1e-12;
  return DLA_SUCCESS;
}

}  // namespace dla

using namespace dla;

extern "C" {

const char* dla_last_error_detail(void) {
  static thread_local char text[160];
  if (tl_hip_error.code == hipSuccess) return "";
  snprintf(text, sizeof(text), "%s (%d) in %s", hipGetErrorName(tl_hip_error.code), (int)tl_hip_error.code,
           tl_hip_error.where);
  return text;
}

const char* dla_version(void) { return "dla-mi355x 0.1 (gfx950, MFMA 16x16x4)"; }

const char* dla_strerror(int code) {
  switch (code) {
    case DLA_SUCCESS: return "success";
    case DLA_ERR_UNSUPPORTED_PARAMS: return "tile/block parameters are not in the pre-instantiated menu";
    case DLA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case DLA_ERR_HIP: return "a HIP call or kernel launch failed";
    case DLA_ERR_TOO_LARGE: return "dimension too large";
    default: return code < 0 ? "invalid argument (its 1-based position is the negated code)" : "unknown error code";
  }
}

int dla_gemm_params_supported(dla_dtype dt, const dla_gemm_params* p) {
  if (dt != DLA_F64 && dt != DLA_F32) return 0;
  GemmSchedule s;
  return resolve_schedule(dt, p, OP_ASSIGN, &s) == DLA_SUCCESS ? 1 : 0;
}

int dla_enumerate_tiles(dla_dtype dt, dla_gemm_params* out, int cap) {
  if (dt != DLA_F64 && dt != DLA_F32) return 0;
  int count = 0;
  for (int i = 0; i < kNumTiles; ++i)
    for (int j = 0; j < kNumKu; ++j) {
      GemmSchedule s = {kTiles[i].tm, kTiles[i].tn, kKu[j].tk, kKu[j].uk, kTiles[i].wm, kTiles[i].wn};
      if (gemm_lds_bytes(s, false, esize(dt)) > kMaxLdsBytes) continue;
      if (out && count < cap) out[count] = dla_gemm_params{s.tm, s.tn, s.tk, s.uk, s.wm, s.wn};
      ++count;
    }
  return count;
}

int dla_block_size_supported(dla_dtype dt, int nb) {
  if (dt != DLA_F64 && dt != DLA_F32) return 0;
  return ((nb >= 16 && nb <= 128 && nb % 16 == 0) || (nb > 128 && nb <= 256 && nb % 32 == 0)) ? 1 : 0;
}

int dla_default_params(int kernel, int64_t n, dla_dtype dt, void* out) {
  if (kernel < DLA_KERNEL_MM3 || kernel > DLA_KERNEL_CHOLESKY) return -1;
  if (n < 0) return -2;
  if (dt != DLA_F64 && dt != DLA_F32) return -3;
  if (!out) return -4;
  if (kernel == DLA_KERNEL_MM3) {
    dla_mm3_params* p = static_cast<dla_mm3_params*>(out);
    GemmSchedule s;
    resolve_schedule(dt, nullptr, OP_ASSIGN, &s, n, n);
    const dla_gemm_params gp = {s.tm, s.tn, s.tk, s.uk, s.wm, s.wn};
    p->e = p->f = p->g = gp;
    return DLA_SUCCESS;
  }
  dla_factor_params* p = static_cast<dla_factor_params*>(out);
  FactorPlan plan;
  GemmSchedule s;
  const int op = kernel == DLA_KERNEL_LU ? OP_SUB : OP_SUB_NT_LOWER;
  int rc = resolve_factor_params(dt, n, nullptr, op, &plan, &s);
  if (rc != DLA_SUCCESS) return rc;
  p->nb = plan.nb_outer;
  p->lookahead = plan.lookahead;
  (void)s;
  p->update = dla_gemm_params{0, 0, 0, 0, 0, 0};  // the panel-stationary update kernel
  p->defer_min_rows = 0;
  return DLA_SUCCESS;
}

int dla_gemm(int op, const void* d_a, int64_t lda, const void* d_b, int64_t ldb, void* d_c, int64_t ldc, int64_t m,
             int64_t n, int64_t k, dla_dtype dt, const dla_gemm_params* p, void* hip_stream) {
  if (op < OP_ASSIGN || op > OP_SUB_TN) return -1;
  if (m < 0) return -8;
  if (n < 0) return -9;
  if (k < 0) return -10;
  if (dt != DLA_F64 && dt != DLA_F32) return -11;
  if (op == OP_SUB_NT_LOWER && m != n) return -9;
  if (m > kMaxDim || n > kMaxDim || k > kMaxDim) return DLA_ERR_TOO_LARGE;
  const bool empty = (m == 0 || n == 0);
  if (!empty && k > 0 && !d_a) return -2;
  if (!empty && k > 0 && !d_b) return -4;
  if (!empty && !d_c) return -6;
  if (lda < (op == OP_SUB_TN ? (m > 0 ? m : 1) : (k > 0 ? k : 1))) return -3;
  if (ldb < ((op == OP_SUB_NT_LOWER || op == OP_SUB_NT) ? (k > 0 ? k : 1) : (n > 0 ? n : 1))) return -5;
  if (ldc < (n > 0 ? n : 1)) return -7;
  const size_t es = (size_t)esize(dt);
  if (((uintptr_t)d_a % es) || ((uintptr_t)d_b % es)) return -2;
  if ((uintptr_t)d_c % es) return -6;
  GemmSchedule s;
  int rc = resolve_schedule(dt, p, op, &s, m, n);
  if (rc != DLA_SUCCESS) return rc;
  hip_clear_stale_error();
  if (op == OP_SUB_TN) {  // instantiated for the 32x32 (16x16 waves) and 64x64 (32x32 waves) macro-tiles only
    if (!p || (p->tile_m == 0 && p->tile_n == 0)) s = GemmSchedule{64, 64, 16, 2, 32, 32};
    const bool ok = (s.tm == 32 && s.tn == 32 && s.wm == 16 && s.wn == 16) || (s.tm == 64 && s.tn == 64 && s.wm == 32 && s.wn == 32);
    if (!ok) return DLA_ERR_UNSUPPORTED_PARAMS;
  }
  if (empty) return DLA_SUCCESS;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (k == 0) {
    if (op != OP_ASSIGN) return DLA_SUCCESS;
    return dt == DLA_F64 ? fill_zero((double*)d_c, ldc, m, n, st) : fill_zero((float*)d_c, ldc, m, n, st);
  }
  if (dt == DLA_F64)
    return run_gemm<double>(s, op, (const double*)d_a, lda, (const double*)d_b, ldb, (double*)d_c, ldc, m, n, k, st);
  return run_gemm<float>(s, op, (const float*)d_a, lda, (const float*)d_b, ldb, (float*)d_c, ldc, m, n, k, st);
}

int dla_rank_update(int lower, const void* d_l, const void* d_r, void* d_c, int64_t ld, int64_t m, int64_t k,
                    dla_dtype dt, void* hip_stream) {
  if (lower != 0 && lower != 1) return -1;
  if (m < 0) return -6;
  if (k < 0 || k > 256) return -7;
  if (dt != DLA_F64 && dt != DLA_F32) return -8;
  if (m > kMaxDim) return DLA_ERR_TOO_LARGE;
  if (m == 0 || k == 0) return DLA_SUCCESS;
  hip_clear_stale_error();
  const size_t es = (size_t)esize(dt);
  if (!d_l || (uintptr_t)d_l % es) return -2;
  if (!lower && (!d_r || (uintptr_t)d_r % es)) return -3;
  if (!d_c || (uintptr_t)d_c % es) return -4;
  if (ld < m || ld < k) return -5;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (dt == DLA_F64)
    return rank_update_impl<double>(lower != 0, (const double*)d_l, (const double*)d_r, (double*)d_c, ld, m, (int)k, st);
  return rank_update_impl<float>(lower != 0, (const float*)d_l, (const float*)d_r, (float*)d_c, ld, m, (int)k, st);
}

size_t dla_mfma_peak_scratch_bytes(void) { return (size_t)kPeakGrid * 256 * sizeof(double); }

int dla_mfma_peak(dla_dtype dt, void* d_scratch, size_t scratch_bytes, void* hip_stream, double* tflops) {
  if (dt != DLA_F64 && dt != DLA_F32) return -1;
  if (!d_scratch || (uintptr_t)d_scratch % 8) return -2;
  if (scratch_bytes < dla_mfma_peak_scratch_bytes()) return DLA_ERR_WORKSPACE;
  if (!tflops) return -5;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  return dt == DLA_F64 ? mfma_peak_impl<double>(d_scratch, st, tflops) : mfma_peak_impl<float>(d_scratch, st, tflops);
}

size_t mm3_workspace_bytes(int64_t ni, int64_t nj, int64_t nl, dla_dtype dt) {
  if (ni < 0 || nj < 0 || nl < 0 || (dt != DLA_F64 && dt != DLA_F32)) return 0;
  if (ni > kMaxDim || nj > kMaxDim || nl > kMaxDim) return 0;
  const Mm3Layout L = mm3_layout(ni, nj, nl, dt);
  return L.e_bytes + L.f_bytes + 256;
}

// Argument checks shared by mm3 and mm3_noalloc (everything but the workspace); resolves the three schedules.
static int mm3_check_args(const void* d_a, int64_t lda, const void* d_b, int64_t ldb, const void* d_c, int64_t ldc,
                          const void* d_d, int64_t ldd, void* d_g, int64_t ldg, int64_t ni, int64_t nk, int64_t nj,
                          int64_t nm, int64_t nl, dla_dtype dt, const dla_mm3_params* p, GemmSchedule* se,
                          GemmSchedule* sf, GemmSchedule* sg) {
  if (ni < 0) return -11;
  if (nk < 0) return -12;
  if (nj < 0) return -13;
  if (nm < 0) return -14;
  if (nl < 0) return -15;
  if (dt != DLA_F64 && dt != DLA_F32) return -16;
  if (ni > kMaxDim || nk > kMaxDim || nj > kMaxDim || nm > kMaxDim || nl > kMaxDim) return DLA_ERR_TOO_LARGE;
  const size_t es = (size_t)esize(dt);
  if (ni > 0 && nk > 0 && (!d_a || (uintptr_t)d_a % es)) return -1;
  if (lda < (nk > 0 ? nk : 1)) return -2;
  if (nk > 0 && nj > 0 && (!d_b || (uintptr_t)d_b % es)) return -3;
  if (ldb < (nj > 0 ? nj : 1)) return -4;
  if (nj > 0 && nm > 0 && (!d_c || (uintptr_t)d_c % es)) return -5;
  if (ldc < (nm > 0 ? nm : 1)) return -6;
  if (nm > 0 && nl > 0 && (!d_d || (uintptr_t)d_d % es)) return -7;
  if (ldd < (nl > 0 ? nl : 1)) return -8;
  if (ni > 0 && nl > 0 && (!d_g || (uintptr_t)d_g % es)) return -9;
  if (ldg < (nl > 0 ? nl : 1)) return -10;
  int rc;
  if ((rc = resolve_schedule(dt, p ? &p->e : nullptr, OP_ASSIGN, se, ni, nj)) != DLA_SUCCESS) return rc;
  if ((rc = resolve_schedule(dt, p ? &p->f : nullptr, OP_ASSIGN, sf, nj, nl)) != DLA_SUCCESS) return rc;
  return resolve_schedule(dt, p ? &p->g : nullptr, OP_ASSIGN, sg, ni, nl);
}

static int mm3_run(const void* d_a, int64_t lda, const void* d_b, int64_t ldb, const void* d_c, int64_t ldc,
                   const void* d_d, int64_t ldd, void* d_g, int64_t ldg, int64_t ni, int64_t nk, int64_t nj, int64_t nm,
                   int64_t nl, dla_dtype dt, const GemmSchedule& se, const GemmSchedule& sf, const GemmSchedule& sg,
                   void* ws, hipStream_t st) {
  hip_clear_stale_error();
  if (dt == DLA_F64)
    return mm3_impl<double>((const double*)d_a, lda, (const double*)d_b, ldb, (const double*)d_c, ldc,
                            (const double*)d_d, ldd, (double*)d_g, ldg, ni, nk, nj, nm, nl, se, sf, sg, ws, st);
  return mm3_impl<float>((const float*)d_a, lda, (const float*)d_b, ldb, (const float*)d_c, ldc, (const float*)d_d,
                         ldd, (float*)d_g, ldg, ni, nk, nj, nm, nl, se, sf, sg, ws, st);
}

int mm3(const void* d_a, int64_t lda, const void* d_b, int64_t ldb, const void* d_c, int64_t ldc, const void* d_d,
        int64_t ldd, void* d_g, int64_t ldg, int64_t ni, int64_t nk, int64_t nj, int64_t nm, int64_t nl,
        dla_dtype dt, const dla_mm3_params* p, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  GemmSchedule se, sf, sg;
  const int rc = mm3_check_args(d_a, lda, d_b, ldb, d_c, ldc, d_d, ldd, d_g, ldg, ni, nk, nj, nm, nl, dt, p, &se, &sf, &sg);
  if (rc != DLA_SUCCESS) return rc;
  const size_t need = mm3_workspace_bytes(ni, nj, nl, dt);
  const bool uses_ws = (ni > 0 && nl > 0 && nj > 0);
  if (uses_ws && (!d_workspace || workspace_bytes < need || (uintptr_t)d_workspace % 256)) return DLA_ERR_WORKSPACE;
  return mm3_run(d_a, lda, d_b, ldb, d_c, ldc, d_d, ldd, d_g, ldg, ni, nk, nj, nm, nl, dt, se, sf, sg, d_workspace,
                 static_cast<hipStream_t>(hip_stream));
}

int mm3_noalloc(const void* d_a, int64_t lda, const void* d_b, int64_t ldb, const void* d_c, int64_t ldc,
                const void* d_d, int64_t ldd, void* d_g, int64_t ldg, int64_t ni, int64_t nk, int64_t nj, int64_t nm,
                int64_t nl, dla_dtype dt, const dla_mm3_params* p, void* hip_stream) {
  GemmSchedule se, sf, sg;
  const int rc = mm3_check_args(d_a, lda, d_b, ldb, d_c, ldc, d_d, ldd, d_g, ldg, ni, nk, nj, nm, nl, dt, p, &se, &sf, &sg);
  if (rc != DLA_SUCCESS) return rc;
  // E and F must fit the fixed scratch
  if (mm3_workspace_bytes(ni, nj, nl, dt) > (size_t)DLA_MM3_NOALLOC_MAX_BYTES) return DLA_ERR_TOO_LARGE;
  void* ws = nullptr;
  if (ni > 0 && nl > 0 && nj > 0) {
    ws = scratch_of_current_device();
    if (!ws) return DLA_ERR_HIP;
  }
  return mm3_run(d_a, lda, d_b, ldb, d_c, ldc, d_d, ldd, d_g, ldg, ni, nk, nj, nm, nl, dt, se, sf, sg, ws,
                 static_cast<hipStream_t>(hip_stream));
}

static int factor_common_checks(void* d_a, int64_t n, int64_t lda, dla_dtype dt) {
  if (n < 0) return -2;
  if (dt != DLA_F64 && dt != DLA_F32) return -4;
  if (n > 0 && !d_a) return -1;
  if (n > 0 && ((uintptr_t)d_a % (size_t)esize(dt))) return -1;
  if (lda < (n > 0 ? n : 1)) return -3;
  if (n > kMaxDim) return DLA_ERR_TOO_LARGE;
  return DLA_SUCCESS;
}

size_t factor_workspace_bytes(int64_t n, dla_dtype dt, const dla_factor_params* p) {
  if (n < 0 || n > kMaxDim || (dt != DLA_F64 && dt != DLA_F32)) return 0;
  return factor_workspace_bytes_impl(n, dt, p);
}

int lu_factor(void* d_a, int64_t n, int64_t lda, dla_dtype dt, const dla_factor_params* p, void* d_workspace,
              size_t workspace_bytes, void* hip_stream, int* d_info) {
  int rc = factor_common_checks(d_a, n, lda, dt);
  if (rc != DLA_SUCCESS) return rc;
  hip_clear_stale_error();
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (dt == DLA_F64) return lu_factor_impl<double>((double*)d_a, n, lda, p, d_workspace, workspace_bytes, st, d_info);
  return lu_factor_impl<float>((float*)d_a, n, lda, p, d_workspace, workspace_bytes, st, d_info);
}

int cholesky_factor(void* d_a, int64_t n, int64_t lda, dla_dtype dt, const dla_factor_params* p, void* d_workspace,
                    size_t workspace_bytes, void* hip_stream, int* d_info) {
  int rc = factor_common_checks(d_a, n, lda, dt);
  if (rc != DLA_SUCCESS) return rc;
  hip_clear_stale_error();
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (dt == DLA_F64)
    return cholesky_factor_impl<double>((double*)d_a, n, lda, p, d_workspace, workspace_bytes, st, d_info);
  return cholesky_factor_impl<float>((float*)d_a, n, lda, p, d_workspace, workspace_bytes, st, d_info);
}

static int solve_common_checks(const void* d_f, int64_t n, int64_t lda, void* d_b, int64_t nrhs, int64_t ldb,
                               dla_dtype dt) {
  if (n < 0) return -2;
  if (nrhs < 0) return -5;
  if (dt != DLA_F64 && dt != DLA_F32) return -7;
  if (n > 0 && (!d_f || ((uintptr_t)d_f % (size_t)esize(dt)))) return -1;
  if (lda < (n > 0 ? n : 1)) return -3;
  if (n > 0 && nrhs > 0 && (!d_b || ((uintptr_t)d_b % (size_t)esize(dt)))) return -4;
  if (ldb < (nrhs > 0 ? nrhs : 1)) return -6;
  if (n > kMaxDim || nrhs > kMaxDim) return DLA_ERR_TOO_LARGE;
  return DLA_SUCCESS;
}

size_t solve_workspace_bytes(int64_t n, int64_t nrhs, dla_dtype dt) {
  if (n < 0 || n > kMaxDim || nrhs < 0 || nrhs > kMaxDim || (dt != DLA_F64 && dt != DLA_F32)) return 0;
  return solve_workspace_bytes_impl(n, nrhs, dt);
}

extern "C++" {
template <int KIND>
static int solve_entry(const void* d_f, int64_t n, int64_t lda, void* d_b, int64_t nrhs, int64_t ldb, dla_dtype dt,
                       void* d_workspace, size_t workspace_bytes, void* hip_stream, int phases) {
  int rc = solve_common_checks(d_f, n, lda, d_b, nrhs, ldb, dt);
  if (rc != DLA_SUCCESS) return rc;
  hip_clear_stale_error();
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (dt == DLA_F64)
    return solve_impl<double, KIND>((const double*)d_f, n, lda, (double*)d_b, nrhs, ldb, d_workspace, workspace_bytes, st, phases);
  return solve_impl<float, KIND>((const float*)d_f, n, lda, (float*)d_b, nrhs, ldb, d_workspace, workspace_bytes, st, phases);
}

template <int KIND>
static int solve_prepare_entry(const void* d_f, int64_t n, int64_t lda, dla_dtype dt, void* d_workspace,
                               size_t workspace_bytes, void* hip_stream) {
  if (n < 0) return -2;
  if (dt != DLA_F64 && dt != DLA_F32) return -4;
  if (n > 0 && (!d_f || ((uintptr_t)d_f % (size_t)esize(dt)))) return -1;
  if (lda < (n > 0 ? n : 1)) return -3;
  if (n > kMaxDim) return DLA_ERR_TOO_LARGE;
  hip_clear_stale_error();
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (dt == DLA_F64)
    return solve_impl<double, KIND>((const double*)d_f, n, lda, nullptr, 0, 1, d_workspace, workspace_bytes, st, kSolvePrepare);
  return solve_impl<float, KIND>((const float*)d_f, n, lda, nullptr, 0, 1, d_workspace, workspace_bytes, st, kSolvePrepare);
}
}  // extern "C++"

int lu_solve(const void* d_lu, int64_t n, int64_t lda, void* d_b, int64_t nrhs, int64_t ldb, dla_dtype dt,
             void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  return solve_entry<0>(d_lu, n, lda, d_b, nrhs, ldb, dt, d_workspace, workspace_bytes, hip_stream, kSolvePrepare | kSolveApply);
}

int cholesky_solve(const void* d_l, int64_t n, int64_t lda, void* d_b, int64_t nrhs, int64_t ldb, dla_dtype dt,
                   void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  return solve_entry<1>(d_l, n, lda, d_b, nrhs, ldb, dt, d_workspace, workspace_bytes, hip_stream, kSolvePrepare | kSolveApply);
}

int lu_solve_prepare(const void* d_lu, int64_t n, int64_t lda, dla_dtype dt, void* d_workspace, size_t workspace_bytes,
                     void* hip_stream) {
  return solve_prepare_entry<0>(d_lu, n, lda, dt, d_workspace, workspace_bytes, hip_stream);
}

int cholesky_solve_prepare(const void* d_l, int64_t n, int64_t lda, dla_dtype dt, void* d_workspace, size_t workspace_bytes,
                           void* hip_stream) {
  return solve_prepare_entry<1>(d_l, n, lda, dt, d_workspace, workspace_bytes, hip_stream);
}

int lu_solve_prepared(const void* d_lu, int64_t n, int64_t lda, void* d_b, int64_t nrhs, int64_t ldb, dla_dtype dt,
                      void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  return solve_entry<0>(d_lu, n, lda, d_b, nrhs, ldb, dt, d_workspace, workspace_bytes, hip_stream, kSolveApply);
}

int cholesky_solve_prepared(const void* d_l, int64_t n, int64_t lda, void* d_b, int64_t nrhs, int64_t ldb, dla_dtype dt,
                            void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  return solve_entry<1>(d_l, n, lda, d_b, nrhs, ldb, dt, d_workspace, workspace_bytes, hip_stream, kSolveApply);
}

int dla_handover_selftest(void* d_scratch, size_t scratch_bytes, void* hip_stream, int* d_info) {
  if (!d_scratch || ((uintptr_t)d_scratch % 256)) return -1;
  if (scratch_bytes < kHandoverSelftestBytes) return -2;
  if (!d_info) return -4;
  hip_clear_stale_error();
  return handover_selftest_impl(d_scratch, static_cast<hipStream_t>(hip_stream), d_info);
}

int dla_profile_enable(int on) {
  std::lock_guard<std::mutex> lock(g_profile_mutex);
  g_profile_on = (on != 0);
  return DLA_SUCCESS;
}

int dla_profile_read(int phase, double* ms_total, int64_t* launches, double* flops) {
  if (phase < 0 || phase >= PHASE_COUNT) return -1;
  std::lock_guard<std::mutex> lock(g_profile_mutex);
  double ms = 0.0, fl = 0.0;
  int64_t cnt = 0;
  std::vector<ProfileRecord> keep;
  for (const ProfileRecord& r : g_records) {
    if (r.phase != phase) {
      keep.push_back(r);
      continue;
    }
    float t = 0.f;
    if (hipEventSynchronize(r.e1) == hipSuccess && hipEventElapsedTime(&t, r.e0, r.e1) == hipSuccess) {
      ms += t;
      fl += r.flops;
      ++cnt;
    }
    g_event_pool.push_back(r.e0);
    g_event_pool.push_back(r.e1);
  }
  g_records.swap(keep);
  if (ms_total) *ms_total = ms;
  if (launches) *launches = cnt;
  if (flops) *flops = fl;
  return DLA_SUCCESS;
}

}  // extern "C"
