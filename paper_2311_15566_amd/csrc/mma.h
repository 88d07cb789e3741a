// Matrix-core product and small device helpers shared by the GEMM kernels.
#pragma once
#include "common.h"

namespace ss {

// one 16 x 16 x FragK product per call: D[n][b] += sum_k W[n][k] * A[b][k]
// lane l returns D[(l>>4)*4 + i][l & 15], i = 0..3
template <typename T> struct Mma;
template <> struct Mma<float> {
  static __device__ __forceinline__ f32x4 mma(u32x4 w, u32x4 a, f32x4 c) {
    f32x4 wf = __builtin_bit_cast(f32x4, w), af = __builtin_bit_cast(f32x4, a);
#pragma unroll
    for (int j = 0; j < 4; ++j) c = __builtin_amdgcn_mfma_f32_16x16x4f32(wf[j], af[j], c, 0, 0, 0);
    return c;
  }
};

// the same product on half-precision operands (bf16 models: weight fragments are stored as halves)
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
__device__ __forceinline__ f32x4 mma_f16(u32x4 w, u32x4 a, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, w), __builtin_bit_cast(f16x8_t, a), c, 0, 0, 0);
}
// the product for a model of element type T: half operands for a 2-byte (bf16) model, float operands otherwise
template <typename T>
__device__ __forceinline__ f32x4 mma_op(u32x4 w, u32x4 a, f32x4 c) {
  if constexpr (sizeof(T) == 2) return mma_f16(w, a, c);
  else return Mma<float>::mma(w, a, c);
}
__device__ __forceinline__ float act_apply(int kind, float h) {
  if (kind == SS_ACT_GELU_TANH) return 0.5f * h * (1.0f + tanhf(0.7978845608028654f * (h + 0.044715f * h * h * h)));
  return fmaxf(h, 0.0f);  // SS_ACT_RELU
}
// Rotary position embedding of one (low, high) pair of a head's dimensions, cs = (cos, sin) of the position's angle for
// that pair.  The order of the operations is spelled out: the kernels of the initial phase that rotate (the q|k|v GEMM's
// epilogue, or prefill_kv_write behind a GEMM that cannot) must agree bit for bit.
__device__ __forceinline__ void rope_rotate(float lo, float hi, float2 cs, float &out_lo, float &out_hi) {
  out_lo = __fmaf_rn(lo, cs.x, -__fmul_rn(hi, cs.y));
  out_hi = __fmaf_rn(lo, cs.y, __fmul_rn(hi, cs.x));
}
__device__ __forceinline__ float silu_f(float g) { return g / (1.0f + __expf(-g)); }
// the same with the hardware's reciprocal (1 ulp) in place of the division: for epilogues that are bound by instruction count
__device__ __forceinline__ float silu_rcp(float g) { return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)); }

// Four consecutive activations (k a multiple of 4) into an operand buffer, as whole 32-bit words.
// DEV: device-scope (write-through) stores, for buffers another block of the same launch reads.
template <typename T, bool DEV>
__device__ __forceinline__ void store4_frag(void *base, int row, int k, int k_blocks, const float (&v)[4]) {
  T w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) w[i] = Elem<T>::from_f32(v[i]);
  uint32_t words[sizeof(T)];  // 4 elements = sizeof(T) words
  __builtin_memcpy(words, w, 4 * sizeof(T));
  uint32_t *p = (uint32_t *)((T *)base + frag_offset<T>(row, k, k_blocks));
#pragma unroll
  for (int i = 0; i < (int)sizeof(T); ++i) {
    if (DEV) st_dev(p + i, words[i]);
    else p[i] = words[i];
  }
}

}  // namespace ss
