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

// Raises a kernel's dynamic-LDS limit once per process (one static instance per kernel instantiation).
// First calls may come from several host threads at the same time.
struct LdsLimitOnce {
  std::once_flag flag;
  hipError_t err = hipSuccess;
  bool ensure(const void* kernel, int bytes) {
    std::call_once(flag, [&] { err = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes); });
    return err == hipSuccess;
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
