// Host-side dispatch of the GEMM kernel menu.  Each macro-tile shape is compiled
// in its own translation unit (gemm_inst_*.hip, generated from gemm_inst.hip.in
// by the build script) so the menu builds in parallel.
#pragma once
#include <hip/hip_runtime.h>
#include <mutex>
#include "gemm_kernel.hpp"

namespace dla {

struct GemmSchedule {
  int tm, tn, tk, uk, wm, wn;
};

constexpr int kMaxLdsBytes = 160 * 1024;  // LDS per CU on gfx950

// Status of the launch just made.  hipGetLastError reports the last error of ANY earlier call of the
// host thread (another library's failed probe included), so every entry point first clears what it
// finds (hip_clear_stale_error) and a launch site then sees only errors of this library's own calls.
// The failing call is kept per host thread for dla_last_error_detail().
struct HipErrorNote {
  const char* where = "";
  hipError_t code = hipSuccess;
};
inline thread_local HipErrorNote tl_hip_error;
inline void hip_clear_stale_error() { (void)hipGetLastError(); }
inline int hip_note(hipError_t e, const char* where) {
  if (e == hipSuccess) return 0;  // DLA_SUCCESS
  tl_hip_error.where = where;
  tl_hip_error.code = e;
  return 3;                       // DLA_ERR_HIP
}
inline int launch_status(const char* where) { return hip_note(hipGetLastError(), where); }

// Raises a kernel's dynamic-LDS limit once per process (one static instance per kernel instantiation).
// First calls may come from several host threads at the same time.
struct LdsLimitOnce {
  std::once_flag flag;
  hipError_t err = hipSuccess;
  bool ensure(const void* kernel, int bytes) {
    std::call_once(flag, [&] { err = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes); });
    return hip_note(err, "hipFuncSetAttribute") == 0;
  }
};

// The macro-tile menu: X(TM, TN, WM, WN).  The first entry with a given
// (TM, TN) is the default wave split for that macro-tile.
#define DLA_TILE_MENU(X) \
  X(16, 16, 16, 16)      \
  X(32, 32, 16, 16)      \
  X(32, 32, 32, 32)      \
  X(64, 64, 32, 32)      \
  X(64, 64, 32, 64)      \
  X(128, 64, 64, 32)     \
  X(64, 128, 32, 64)     \
  X(128, 128, 64, 64)    \
  X(128, 128, 32, 64)    \
  X(256, 128, 64, 64)    \
  X(128, 256, 64, 64)

// k-slab depths and unroll factors instantiated for every macro-tile: X(TK, UK)
#define DLA_KU_MENU(X) X(8, 1) X(8, 2) X(16, 1) X(16, 2) X(16, 4) X(32, 2) X(32, 4) X(32, 8) X(128, 8)

// Completion event for the NEXT GEMM launch of this host thread (consumed and cleared by that
// launch): it rides on the kernel's dispatch packet instead of a marker packet behind it.
inline thread_local hipEvent_t tl_gemm_done_event = nullptr;

template <typename T, int TM, int TN, int WM, int WN>
int launch_gemm_tile(const GemmSchedule& s, int op, const GemmGroup<T>& g, hipStream_t st);

// Returns DLA_SUCCESS, DLA_ERR_UNSUPPORTED_PARAMS or DLA_ERR_HIP.
template <typename T>
int launch_gemm(const GemmSchedule& s, int op, const GemmGroup<T>& g, hipStream_t st);

// LDS bytes of a schedule (both dtypes share the formula), used for menu legality on the host.
inline int gemm_lds_bytes(const GemmSchedule& s, bool bt, int esz) {
  const int sa = s.tk + 1, sb = bt ? s.tk + 1 : s.tn;
  const int al = 16 / esz;
  const int a = (s.tm * sa + al - 1) / al * al;
  const int b = ((bt ? s.tn * sb : s.tk * sb) + al - 1) / al * al;
  return 2 * (a + b) * esz;
}

}  // namespace dla
