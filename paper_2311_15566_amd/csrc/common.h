// Shared declarations of the spotshard HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stdio.h>
#include <string>
#include <vector>
#include <map>
#include <set>

#include "../../include/spotshard.h"

namespace ss {

// ---------------------------------------------------------------------------
// error plumbing
// ---------------------------------------------------------------------------
void set_error(const char *fmt, ...);
#define SS_FAIL(code, ...)        \
  do {                            \
    ::ss::set_error(__VA_ARGS__); \
    return (code);                \
  } while (0)
#define SS_HIP(call)                                                                   \
  do {                                                                                 \
    hipError_t e_ = (call);                                                            \
    if (e_ != hipSuccess) SS_FAIL(SS_EHIP, "%s: %s", #call, hipGetErrorString(e_));    \
  } while (0)
#define SS_TRY(call)                  \
  do {                                \
    ss_status s_ = (call);            \
    if (s_ != SS_OK) return s_;       \
  } while (0)

// ---------------------------------------------------------------------------
// Launch of a decode-step kernel.  In measurement mode the caller leaves a pair of events here
// and the launch records the kernel's own begin and end on them (the dispatch's timestamps, as
// a profiler sees them, with no marker packets between kernels).
// ---------------------------------------------------------------------------
struct LaunchTiming {
  hipEvent_t start = nullptr, stop = nullptr;
};
extern thread_local LaunchTiming g_launch_timing;
#define SS_LAUNCH_KERNEL(kern, grid, block, lds, st, ...)                                                           \
  do {                                                                                                              \
    if (::ss::g_launch_timing.start)                                                                                \
      hipExtLaunchKernelGGL(kern, grid, block, lds, st, ::ss::g_launch_timing.start, ::ss::g_launch_timing.stop, 0, \
                            __VA_ARGS__);                                                                           \
    else                                                                                                            \
      hipLaunchKernelGGL(kern, grid, block, lds, st, __VA_ARGS__);                                                  \
  } while (0)

// ---------------------------------------------------------------------------
// element types
// ---------------------------------------------------------------------------
typedef uint16_t bf16_t;  // bfloat16 bit pattern
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__host__ __device__ inline float bf16_to_f32(bf16_t b) {
  union { uint32_t u; float f; } c;
  c.u = ((uint32_t)b) << 16;
  return c.f;
}
// round-to-nearest-even; inputs are finite
__host__ __device__ inline bf16_t f32_to_bf16(float f) {
  union { uint32_t u; float f; } c;
  c.f = f;
  uint32_t u = c.u;
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

typedef _Float16 f16_t;   // IEEE half: a KV-cache element type
template <typename T> struct Elem;
template <> struct Elem<f16_t> {
  static constexpr int kPerLane = 8;
  static constexpr int kFragK = 32;
  __host__ __device__ static float to_f32(f16_t v) { return (float)v; }
  // round-to-nearest-even, saturating at the largest finite half
  __host__ __device__ static f16_t from_f32(float v) {
    v = v > 65504.f ? 65504.f : (v < -65504.f ? -65504.f : v);
    return (f16_t)v;
  }
};
template <> struct Elem<float> {
  static constexpr int kPerLane = 4;   // elements in a lane's 16-byte piece
  static constexpr int kFragK = 16;    // k extent of one 1 KiB operand fragment
  __host__ __device__ static float to_f32(float v) { return v; }
  __host__ __device__ static float from_f32(float v) { return v; }
};
template <> struct Elem<bf16_t> {
  static constexpr int kPerLane = 8;
  static constexpr int kFragK = 32;
  // (activations of bf16 models are never stored as bf16: 8 significant bits miss the logits bar on
  // the larger shapes; the GEMM operands are halves, see Operand)
  __host__ __device__ static float to_f32(bf16_t v) { return bf16_to_f32(v); }
  __host__ __device__ static bf16_t from_f32(float v) { return f32_to_bf16(v); }
};

// Matrix-core operand order.  A [rows x K] operand (weights: rows = output features;
// activations: rows = batch rows / tokens) is stored as 1 KiB fragments
// [row_tile = rows/16][k_block = K/FragK][lane 0..63][PerLane], where lane = (kq*16 + r)
// holds row r of the tile and the k's  k_block*FragK + kq*PerLane + (0..PerLane-1).
// Both operands of a product use the same order, so a wave loads one fragment as one
// fully coalesced 1 KiB access and the k permutation cancels in the dot product.
template <typename T>
__host__ __device__ inline size_t frag_offset(int row, int k, int k_blocks) {
  constexpr int PL = Elem<T>::kPerLane, FK = Elem<T>::kFragK;
  size_t frag = (size_t)(row >> 4) * k_blocks + (k / FK);
  int kk = k % FK;
  int lane = (kk / PL) * 16 + (row & 15);
  return frag * (64 * PL) + lane * PL + (kk % PL);
}

// ---------------------------------------------------------------------------
// Cross-block hand-off inside one kernel without whole-cache write-backs.  Each XCD has its
// own L2, so data one block leaves for another goes through device-scope (write-through /
// read-around) accesses; the writer waits for its stores to complete, the block then bumps a
// device-scope counter, and whoever sees the final count reads with device-scope loads.
// ---------------------------------------------------------------------------
#ifdef __HIPCC__
__device__ __forceinline__ void st_dev(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(int *p, int v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(uint32_t *p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_dev(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int ld_dev(const int *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Single-assignment rule: a buffer that one block writes and another block of the SAME launch
// reads with ordinary (L2-cached) loads is written with st_dev and is written only once per
// launch, at an address no block has read earlier in that launch; then no L2 can hold a stale
// copy of it.  Buffers that are rewritten within a launch (partials, counters) are read with
// ld_dev.

// Called by every thread of the block after its st_dev stores.  Returns true in every thread
// of the one block that arrives last of `expected`; that block also re-arms the counter.
__device__ __forceinline__ bool arrive_last(int *counter, int expected, int *s_flag) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0) {
    const int old = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = old == expected - 1;
    if (last) st_dev(counter, 0);
    *s_flag = last;
  }
  __syncthreads();
  return *s_flag != 0;
}
#endif

// four consecutive cache elements (one 8- or 16-byte store) from four floats
template <typename T>
__device__ __forceinline__ void store4_cache(T *dst, const f32x4 &v) {
  T t[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) t[i] = Elem<T>::from_f32(v[i]);
  if constexpr (sizeof(T) == 2) {
    uint2 raw;
    __builtin_memcpy(&raw, t, 8);
    *(uint2 *)dst = raw;
  } else {
    *(f32x4 *)dst = v;
  }
}

// store a float activation into an operand buffer
template <typename T>
__device__ inline void store_act(void *base, int row, int k, int k_blocks, float v) {
  ((T *)base)[frag_offset<T>(row, k, k_blocks)] = Elem<T>::from_f32(v);
}

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline size_t align_up(size_t a, size_t b) { return (a + b - 1) / b * b; }

// ---------------------------------------------------------------------------
// device-side view of one layer and of the shard
// ---------------------------------------------------------------------------
struct LayerDev {
  const float *ln1_g, *ln1_b, *ln2_g, *ln2_b;
  const void *wqkv;  // fragments, rows = [q heads | k heads | v heads] x Dh, K = d
  const float *bqkv;
  const void *wo;    // rows = d, K = Hs*Dh
  const float *bo;
  const void *w1;    // rows = Fs (SwiGLU: gate/up fragment rows interleaved per 16-row tile, 2*Fs), K = d
  const float *b1;
  const void *w2;    // rows = d, K = Fs
  const float *b2;
};

struct Shard;  // defined in shard.h

}  // namespace ss
