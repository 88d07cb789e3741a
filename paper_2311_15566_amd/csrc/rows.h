// Row-wise device helpers: block reductions, the embedding of one row, norm statistics.
#pragma once
#include "kernels.h"

namespace ss {

// sum over a 256-thread block; every thread gets the result.  scratch: 4 floats of LDS.
__device__ __forceinline__ float block_sum(float v, float *scratch) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) v += __shfl_xor(v, off);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
  __syncthreads();
  return scratch[0] + scratch[1] + scratch[2] + scratch[3];
}

template <typename T>
__device__ __forceinline__ void widen16(const u32x4 &raw, float *out);
template <>
__device__ __forceinline__ void widen16<float>(const u32x4 &raw, float *out) {
  f32x4 f = __builtin_bit_cast(f32x4, raw);
  out[0] = f[0], out[1] = f[1], out[2] = f[2], out[3] = f[3];
}
template <>
__device__ __forceinline__ void widen16<bf16_t>(const u32x4 &raw, float *out) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[2 * i] = __uint_as_float(raw[i] << 16);
    out[2 * i + 1] = __uint_as_float(raw[i] & 0xffff0000u);
  }
}

// PL consecutive activations (k a multiple of PL) of row `row` as the lane's 16-byte piece of an operand fragment
template <typename OT>
__device__ __forceinline__ void store_piece(void *base, int row, int k, int k_blocks, const float *y) {
  constexpr int PL = Elem<OT>::kPerLane;
  OT h[PL];
#pragma unroll
  for (int e = 0; e < PL; ++e) h[e] = Elem<OT>::from_f32(y[e]);
  u32x4 w;
  __builtin_memcpy(&w, h, 16);
  *(u32x4 *)((OT *)base + frag_offset<OT>(row, k, k_blocks)) = w;
}

// x[r] = wte[token] (+ wpe[position]) with 16-byte loads (or the previous stage's hidden row), d <= 16384,
// and the first GEMM's operand, centred on the row's mean c (RMSNorm: c = 0): (x - c) * gamma as
// fragments of OT elements, with the centred sums (sum (x-c), sum (x-c)^2) and c itself where the
// caller asks for them (decode step: stat_out, cen_out; initial phase: pstat_out, mr_out).
template <typename T>
__device__ __forceinline__ void embed_row_block(const EmbedArgs &a, const int r, float *scratch) {
  typedef typename Operand<T>::type OT;
  constexpr int PL = Elem<T>::kPerLane, FK = Elem<T>::kFragK, MAXV = 64 / PL;
  static_assert(Elem<OT>::kPerLane == PL && Elem<OT>::kFragK == FK, "operand and weight fragments have one geometry");
  int tok = a.hidden ? 0 : a.tokens[r];
  tok = min(max(tok, 0), a.V - 1);
  int pos = a.lens ? a.lens[r] : (r % a.S);
  if (a.wpe) pos = min(pos, a.max_pos - 1);
  const int nvec = a.d / PL;
  const u32x4 *te = (const u32x4 *)((const T *)a.wte + (size_t)tok * a.d);
  const u32x4 *pe = (a.wpe && !a.hidden) ? (const u32x4 *)((const T *)a.wpe + (size_t)pos * a.d) : nullptr;
  float vals[MAXV][PL];
  float s1 = 0.f;
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int v = threadIdx.x + i * 256;
    if (v < nvec) {
      if (a.hidden) {
#pragma unroll
        for (int e = 0; e < PL; ++e) vals[i][e] = a.hidden[(size_t)r * a.d + (size_t)v * PL + e];
      } else {
        widen16<T>(te[v], vals[i]);
      }
      if (pe) {
        float p[PL];
        widen16<T>(pe[v], p);
#pragma unroll
        for (int e = 0; e < PL; ++e) vals[i][e] += p[e];
      }
      float *xo = a.x + (size_t)r * a.d + (size_t)v * PL;
#pragma unroll
      for (int e = 0; e < PL; ++e) {
        s1 += vals[i][e];
        xo[e] = vals[i][e];
      }
    }
  }
  if (!a.act_out) return;
  const float c = a.rms ? 0.f : block_sum(s1, scratch) / (float)a.d;
  float s2 = 0.f;
  s1 = 0.f;
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int v = threadIdx.x + i * 256;
    if (v < nvec) {
      float y[PL];
#pragma unroll
      for (int e = 0; e < PL; ++e) {
        const float t = vals[i][e] - c;
        s1 += t, s2 += t * t;
        y[e] = t * a.gamma[v * PL + e];
      }
      store_piece<OT>(a.act_out, r, v * PL, a.d / FK, y);
      if (a.act_lo_out) {
        float lo[PL];
#pragma unroll
        for (int e = 0; e < PL; ++e) lo[e] = y[e] - Elem<OT>::to_f32(Elem<OT>::from_f32(y[e]));
        store_piece<OT>(a.act_lo_out, r, v * PL, a.d / FK, lo);
      }
    }
  }
  s1 = block_sum(s1, scratch);
  s2 = block_sum(s2, scratch);
  if (threadIdx.x == 0) {
    if (a.stat_out) ((f32x4 *)a.stat_out)[r] = f32x4{s1, s2, 0.f, 0.f};
    if (a.cen_out) a.cen_out[r] = c;
    if (a.pstat_out) a.pstat_out[r] = make_float2(s1, s2);
    if (a.mr_out) a.mr_out[r] = f32x4{c, 0.f, 0.f, 0.f};
  }
}

}  // namespace ss
