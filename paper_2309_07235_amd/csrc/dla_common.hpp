// Shared device-side definitions of the HIP kernels: MFMA wrappers and the
// register layouts of the 16x16x4 matrix instructions on gfx950.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

namespace dla {

typedef double double4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef double double2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// One 16x16x4 MFMA step  D(16x16) = A(16x4) * B(4x16) + C  on a 64-lane wavefront.
// Operand layouts (checked against the hardware with a register-dump probe):
//   A: lane l holds A[l % 16][l / 16]          B: lane l holds B[l / 16][l % 16]
//   D, fp64: register v of lane l holds D[4*v + l/16][l % 16]
//   D, fp32: register v of lane l holds D[4*(l/16) + v][l % 16]
// The fp64 D layout is the B layout of k-step v, so a result block can be fed
// back as the right-hand operand of a following product without a shuffle.
template <typename T>
struct Mfma;

template <>
struct Mfma<double> {
  using acc_t = double4_t;
  using vec2_t = double2_t;
  __device__ static inline acc_t mma(double a, double b, acc_t c) {
    return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
  }
  __device__ static inline int row_of(int v, int lane) { return 4 * v + (lane >> 4); }
};

template <>
struct Mfma<float> {
  using acc_t = float4_t;
  using vec2_t = float2_t;
  __device__ static inline acc_t mma(float a, float b, acc_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
  }
  __device__ static inline int row_of(int v, int lane) { return 4 * (lane >> 4) + v; }
};

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every global load
// and store in flight (its fence covers all address spaces), which would serialise the prefetches
// these kernels keep running across barriers.
__device__ inline void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Hand-over between two kernels that run side by side on different streams: the producer's
// threads make their stores visible device-wide and one of them bumps a counter; the consumer polls
// the counter with one thread before it touches the data.  The consumer is launched early only to
// hide its launch latency; the streams are arranged so that the producer never depends on the
// consumer.  The poll is bounded by the constant-rate wall clock (budget_ticks of it, sized on the
// host from the longest kernel the producer may be queued behind), so that every wave exits even
// where kernels of one process cannot run side by side (a profiler or debugger that serialises
// them): the consumer that gives up sets *broken, every later wait returns at once, and the
// pipeline's last kernel reports it.  Data computed after that is not valid.
// The device-scope release and acquire are each done by ONE thread: they write back and invalidate
// caches that all waves of the workgroup share, and the workgroup barrier next to them orders the
// other waves' stores before the release and their loads after the acquire.  (Issued by every wave,
// the same fences take about a microsecond longer per hand-over.)
__device__ inline void chain_signal(int* counter, int add, int tid) {
  __syncthreads();   // every wave's global stores have been performed for the workgroup
  if (tid == 0) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    __hip_atomic_fetch_add(counter, add, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}
__device__ inline void chain_wait(const int* counter, int target, int* broken, long long budget_ticks, int tid) {
  if (tid == 0) {
    bool ok = __hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target;
    if (!ok) {
      const long long t0 = wall_clock64();
      for (int spins = 0; !ok && spins < (1 << 24); ++spins) {  // the spin cap is a second, absolute bound
        __builtin_amdgcn_s_sleep(16);
        ok = __hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target;
        if (!ok && (spins & 63) == 63) {
          if (__hip_atomic_load(broken, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) break;
          if (wall_clock64() - t0 > budget_ticks) break;
        }
      }
    }
    if (!ok) __hip_atomic_store(broken, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // loads below see what the producer published
  }
  __syncthreads();
}

constexpr int kNumXcd = 8;  // MI355X: 8 accelerator complex dies, workgroups are dealt round-robin

// Workgroup id -> logical work item so that each XCD (and its private L2)
// walks one contiguous range of the work list.
__device__ inline int xcd_contiguous_id(int bid, int total) {
  const int q = total / kNumXcd, r = total % kNumXcd;
  const int x = bid % kNumXcd, t = bid / kNumXcd;
  return x * q + (x < r ? x : r) + t;
}

}  // namespace dla
