// Attention kernels: sequence-split decode attention over the committed KV cache with the
// append of the new token fused in, and the causal attention of the initial phase.
#include "attn_block.h"
#include "kernels.h"

#include <math.h>

namespace ss {

template <typename T, typename AT, int DH, int NWV>
__global__ void __launch_bounds__(NWV * 64) decode_attn(DecodeAttnArgs a) {
  __shared__ AttnShared<NWV> sh;
  decode_attn_block<T, AT, DH, NWV>(a, blockIdx.x, blockIdx.y, sh);
}

ss_status check_decode_attn(const DecodeAttnArgs &a) {
  if (a.B < 1 || a.B > 32 || a.Hs < 1 || (a.Dh != 64 && a.Dh != 128)) SS_FAIL(SS_EINVAL, "decode attention: bad shape");
  if (a.waves != 4 && a.waves != 16) SS_FAIL(SS_EINVAL, "decode attention: %d waves per block", a.waves);
  if (a.rows_per_block < 1 || a.splits < 1 || (size_t)a.splits * a.rows_per_block < (size_t)a.Smax)
    SS_FAIL(SS_EINVAL, "decode attention: %d splits of %d rows do not cover %d rows", a.splits, a.rows_per_block, a.Smax);
  return SS_OK;
}

ss_status launch_decode_attn(int dtype, const DecodeAttnArgs &a, hipStream_t st) {
  SS_TRY(check_decode_attn(a));
  dim3 grid(a.B * a.Hs, a.splits);
#define SS_LAUNCH(KT, AT, DH)                                                                        \
  do {                                                                                               \
    if (a.waves == 16) SS_LAUNCH_KERNEL((decode_attn<KT, AT, DH, 16>), grid, dim3(1024), 0, st, a); \
    else SS_LAUNCH_KERNEL((decode_attn<KT, AT, DH, 4>), grid, dim3(256), 0, st, a);                \
  } while (0)
  if (dtype == SS_DTYPE_BF16 && a.kv_dtype == SS_DTYPE_F16) {
    if (a.Dh == 128) SS_LAUNCH(f16_t, bf16_t, 128);
    else SS_LAUNCH(f16_t, bf16_t, 64);
  } else if (dtype == SS_DTYPE_BF16 && a.kv_dtype == SS_DTYPE_BF16) {
    if (a.Dh == 128) SS_LAUNCH(bf16_t, bf16_t, 128);
    else SS_LAUNCH(bf16_t, bf16_t, 64);
  } else if (dtype == SS_DTYPE_F32 && a.kv_dtype == SS_DTYPE_F32) {
    if (a.Dh == 128) SS_LAUNCH(float, float, 128);
    else SS_LAUNCH(float, float, 64);
  } else {
    SS_FAIL(SS_EINVAL, "decode attention: dtype %d with kv_dtype %d", dtype, a.kv_dtype);
  }
#undef SS_LAUNCH
  SS_HIP(hipGetLastError());
  return SS_OK;
}

// ---------------------------------------------------------------------------
// initial phase: rotate q (in place) and k, write K/V rows of all prompt positions
// grid = (T tokens, Hs); block = DH threads
// ---------------------------------------------------------------------------
template <typename T, int DH>
__global__ void __launch_bounds__(DH) prefill_kv_write(PrefillAttnArgs a) {
  const int t = blockIdx.x, h = blockIdx.y, e = threadIdx.x;
  const int b = t / a.S, pos = t - b * a.S;
  const int HD = a.Hs * DH;
  float *row = a.qkv + (size_t)t * 3 * HD;
  const float2 *tab = a.rope ? a.rope + (size_t)pos * (DH / 2) : nullptr;
  const float q = rope_elem(row + h * DH, e, DH / 2, tab);
  const float k = rope_elem(row + HD + h * DH, e, DH / 2, tab);
  const float v = row[2 * HD + h * DH + e];
  __syncthreads();  // every thread has read its pair before q is overwritten
  row[h * DH + e] = q;
  const size_t off = b * a.row_stride + h * a.head_stride + (size_t)pos * DH * sizeof(T);
  ((T *)(a.k_cache + off))[e] = Elem<T>::from_f32(k);
  ((T *)(a.v_cache + off))[e] = Elem<T>::from_f32(v);
}

ss_status launch_prefill_kv_write(int dtype, const PrefillAttnArgs &a, hipStream_t st) {
  if (a.S < 1 || a.S > a.Smax || a.B < 1 || (a.Dh != 64 && a.Dh != 128)) SS_FAIL(SS_EINVAL, "prefill KV write: bad shape");
  dim3 grid(a.B * a.S, a.Hs);
#define SS_LAUNCH(KT, DH) hipLaunchKernelGGL((prefill_kv_write<KT, DH>), grid, dim3(DH), 0, st, a)
  (void)dtype;
  if (a.kv_dtype == SS_DTYPE_F16) {
    if (a.Dh == 128) SS_LAUNCH(f16_t, 128);
    else SS_LAUNCH(f16_t, 64);
  } else if (a.kv_dtype == SS_DTYPE_BF16) {
    if (a.Dh == 128) SS_LAUNCH(bf16_t, 128);
    else SS_LAUNCH(bf16_t, 64);
  } else {
    if (a.Dh == 128) SS_LAUNCH(float, 128);
    else SS_LAUNCH(float, 64);
  }
#undef SS_LAUNCH
  SS_HIP(hipGetLastError());
  return SS_OK;
}

// ---------------------------------------------------------------------------
// causal attention of the initial phase.  grid = (B*Hs, ceil(S/64)); block = 256 threads:
// thread (qi = tid/4, part = tid%4) owns a quarter of the head dims of query qi.  Keys and
// values (read back from the cache, i.e. at cache precision) go through LDS 32 rows at a time.
// ---------------------------------------------------------------------------
template <typename T, typename AT, int DH>
__global__ void __launch_bounds__(256) prefill_attn(PrefillAttnArgs a) {
  constexpr int TQ = 64, TK = 32, DP = DH / 4, EPL = Elem<T>::kPerLane;
  __shared__ __align__(16) float sk[TK][DH + 4];
  __shared__ __align__(16) float sv[TK][DH + 4];
  const int tid = threadIdx.x;
  const int bh = blockIdx.x, qt = blockIdx.y;
  const int b = bh / a.Hs, h = bh - b * a.Hs;
  const int HD = a.Hs * DH;
  const int qi = qt * TQ + (tid >> 2), part = tid & 3;
  const bool qlive = qi < a.S;
  const float scale = rsqrtf((float)DH);
  float q[DP], acc[DP];
  const float *qrow = a.qkv + ((size_t)(b * a.S + (qlive ? qi : 0))) * 3 * HD + h * DH + part * DP;
#pragma unroll
  for (int e = 0; e < DP; ++e) q[e] = qrow[e], acc[e] = 0.f;
  float m = -1e30f, l = 0.f;
  const char *kbase = a.k_cache + b * a.row_stride + h * a.head_stride;
  const char *vbase = a.v_cache + b * a.row_stride + h * a.head_stride;
  const int last_key = min(a.S, (qt + 1) * TQ);  // keys beyond the tile's last query are never needed
  constexpr int PIECES = DH / EPL;               // 16-byte pieces per row
  for (int k0 = 0; k0 < last_key; k0 += TK) {
    __syncthreads();
    for (int i = tid; i < TK * PIECES; i += 256) {
      const int r = i / PIECES, p = i - r * PIECES;
      const int kr = min(k0 + r, a.S - 1);
      float f[EPL];
      unpack16<T>(*((const u32x4 *)(kbase + (size_t)kr * DH * sizeof(T)) + p), f);
#pragma unroll
      for (int e = 0; e < EPL; ++e) sk[r][p * EPL + e] = f[e];
      unpack16<T>(*((const u32x4 *)(vbase + (size_t)kr * DH * sizeof(T)) + p), f);
#pragma unroll
      for (int e = 0; e < EPL; ++e) sv[r][p * EPL + e] = f[e];
    }
    __syncthreads();
    const int kend = min(TK, last_key - k0);
    for (int j = 0; j < kend; ++j) {
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < DP; ++e) d += q[e] * sk[j][part * DP + e];
      d += __shfl_xor(d, 1);
      d += __shfl_xor(d, 2);
      if (k0 + j <= qi) {  // causal mask
        const float s = d * scale;
        const float mn = fmaxf(m, s);
        const float alpha = __expf(m - mn), p = __expf(s - mn);
        l = l * alpha + p;
#pragma unroll
        for (int e = 0; e < DP; ++e) acc[e] = acc[e] * alpha + p * sv[j][part * DP + e];
        m = mn;
      }
    }
  }
  if (qlive) {
    const float inv = 1.0f / l;
    const int tok = b * a.S + qi;
#pragma unroll
    for (int e = 0; e < DP; ++e)
      store_act<AT>(a.o_out, tok, h * DH + part * DP + e, HD / Elem<AT>::kFragK, Elem<AT>::kParts, acc[e] * inv);
  }
}

ss_status launch_prefill_attn(int dtype, const PrefillAttnArgs &a, hipStream_t st) {
  if (a.S < 1 || a.S > a.Smax || a.B < 1 || (a.Dh != 64 && a.Dh != 128)) SS_FAIL(SS_EINVAL, "prefill attention: bad shape");
  dim3 grid(a.B * a.Hs, ceil_div(a.S, 64));
#define SS_LAUNCH(KT, AT, DH) hipLaunchKernelGGL((prefill_attn<KT, AT, DH>), grid, dim3(256), 0, st, a)
  if (dtype == SS_DTYPE_BF16 && a.kv_dtype == SS_DTYPE_F16) {
    if (a.Dh == 128) SS_LAUNCH(f16_t, bf16_t, 128);
    else SS_LAUNCH(f16_t, bf16_t, 64);
  } else if (dtype == SS_DTYPE_BF16 && a.kv_dtype == SS_DTYPE_BF16) {
    if (a.Dh == 128) SS_LAUNCH(bf16_t, bf16_t, 128);
    else SS_LAUNCH(bf16_t, bf16_t, 64);
  } else if (dtype == SS_DTYPE_F32 && a.kv_dtype == SS_DTYPE_F32) {
    if (a.Dh == 128) SS_LAUNCH(float, float, 128);
    else SS_LAUNCH(float, float, 64);
  } else {
    SS_FAIL(SS_EINVAL, "prefill attention: dtype %d with kv_dtype %d", dtype, a.kv_dtype);
  }
#undef SS_LAUNCH
  SS_HIP(hipGetLastError());
  return SS_OK;
}

}  // namespace ss
