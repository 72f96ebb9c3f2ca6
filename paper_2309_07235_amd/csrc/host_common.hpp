// Host-side helpers shared by the C-ABI entry points: schedule resolution,
// GEMM problem descriptors and the optional per-phase event profiler.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "dla_codes.hpp"
#include "gemm_dispatch.hpp"

namespace dla {

enum Phase { PHASE_GEMM = 0, PHASE_DIAG = 1, PHASE_TRSM = 2, PHASE_UPDATE = 3, PHASE_COUNT = 4 };

// Fills defaults into a user schedule and checks it against the menu.
// op selects which LDS layout the fit check uses.
// m, n (optional): the output size, used to pick the default macro-tile when the caller names none.
int resolve_schedule(dla_dtype dt, const dla_gemm_params* in, int op, GemmSchedule* out, int64_t m = 0,
                     int64_t n = 0);

template <typename T>
inline GemmProblem<T> make_problem(const GemmSchedule& s, int op, const T* A, int64_t lda, const T* B, int64_t ldb,
                                   T* C, int64_t ldc, int64_t M, int64_t N, int64_t K, int tile_begin) {
  GemmProblem<T> p;
  p.A = A;
  p.B = B;
  p.C = C;
  p.lda = lda;
  p.ldb = ldb;
  p.ldc = ldc;
  p.M = (int)M;
  p.N = (int)N;
  p.K = (int)K;
  p.tiles_m = (int)((M + s.tm - 1) / s.tm);
  p.tiles_n = (int)((N + s.tn - 1) / s.tn);
  p.tile_begin = tile_begin;
  p.C2 = nullptr;
  p.ldc2 = 0;
  return p;
}

template <typename T>
inline int problem_tiles(const GemmSchedule& s, int op, const GemmProblem<T>& p) {
  if (op == OP_SUB_NT_LOWER && s.tm == s.tn) return p.tiles_m * (p.tiles_m + 1) / 2;
  return p.tiles_m * p.tiles_n;
}

// One GEMM on a stream (C op= A*B), with profiling brackets when enabled.
template <typename T>
int run_gemm(const GemmSchedule& s, int op, const T* A, int64_t lda, const T* B, int64_t ldb, T* C, int64_t ldc,
             int64_t M, int64_t N, int64_t K, hipStream_t st);

// Profiler brackets: begin returns a slot (or -1 when profiling is off).
int profile_begin(int phase, double flops, hipStream_t st);
void profile_end(int slot, hipStream_t st);

// For a launch that can carry its own start / stop events (hipExtLaunchKernelGGL): a record whose two
// events the caller attaches to the kernel's dispatch, so that the record holds the kernel's own
// duration, as a kernel trace reports it.  False when profiling is off.
bool profile_kernel_events(int phase, double flops, hipEvent_t* start, hipEvent_t* stop);

struct ProfileScope {
  int slot;
  hipStream_t st;
  ProfileScope(int phase, double flops, hipStream_t s) : slot(profile_begin(phase, flops, s)), st(s) {}
  ~ProfileScope() { profile_end(slot, st); }
};

// Factorisation drivers (factor.hip).
template <typename T>
int lu_factor_impl(T* A, int64_t n, int64_t lda, const dla_factor_params* p, void* ws, size_t ws_bytes,
                   hipStream_t st, int* d_info);
template <typename T>
int cholesky_factor_impl(T* A, int64_t n, int64_t lda, const dla_factor_params* p, void* ws, size_t ws_bytes,
                         hipStream_t st, int* d_info);
// The bulk trailing-update kernel on its own: C (m x m) -= L (m x b) * R (b x m), or lower(C) -= L * L^T.
template <typename T>
int rank_update_impl(bool lower, const T* L, const T* Rm, T* C, int64_t ld, int64_t m, int b, hipStream_t st);
// Solve with the factors (solve.hip); KIND is FactorKind as an int; phases: which of its two parts to run.
constexpr int kSolvePrepare = 1, kSolveApply = 2;
template <typename T, int KIND>
int solve_impl(const T* F, int64_t n, int64_t lda, T* B, int64_t nrhs, int64_t ldb, void* ws, size_t ws_bytes,
               hipStream_t st, int phases);
size_t solve_workspace_bytes_impl(int64_t n, int64_t nrhs, dla_dtype dt);
size_t factor_workspace_bytes_impl(int64_t n, dla_dtype dt, const dla_factor_params* p);
constexpr size_t kHandoverSelftestBytes = 8192;
int handover_selftest_impl(void* scratch, hipStream_t st, int* d_info);
// What a dla_factor_params resolves to.  nb: the width of the sub-panel one diagonal-block kernel factors
// (= nb_outer up to 128, else half of it); two_level: bulk updates may run two sub-panels deep, while the
// trailing matrix has at least defer_min_rows rows.
struct FactorPlan {
  int nb_outer, nb, lookahead;
  bool two_level;
  int64_t defer_min_rows;
};
int resolve_factor_params(dla_dtype dt, int64_t n, const dla_factor_params* in, int op, FactorPlan* plan,
                          GemmSchedule* upd);

}  // namespace dla
