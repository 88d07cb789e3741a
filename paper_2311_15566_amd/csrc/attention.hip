// Attention kernels: sequence-split decode attention over the committed KV cache with the
// append of the new token fused in, and the causal attention of the initial phase.
#include "attn_block.h"
#include "kernels.h"
#include "mma.h"

#include <math.h>

namespace ss {

// (8-wave blocks are meant to sit two to a compute unit: four waves a SIMD, at most 128 registers)
template <typename T, typename AT, int DH, int NWV, bool RAW>
__global__ void __launch_bounds__(NWV * 64, NWV == 8 ? 4 : 1) decode_attn(DecodeAttnArgs a) {
  __shared__ AttnShared<NWV> sh;
  decode_attn_block<T, AT, DH, NWV, RAW>(a, blockIdx.x, blockIdx.y, sh);
}

ss_status check_decode_attn(const DecodeAttnArgs &a) {
  if (a.B < 1 || a.B > 32 || a.Hs < 1 || (a.Dh != 64 && a.Dh != 128)) SS_FAIL(SS_EINVAL, "decode attention: bad shape");
  if (a.waves != 4 && a.waves != 8 && a.waves != 16) SS_FAIL(SS_EINVAL, "decode attention: %d waves per block", a.waves);
  if (a.norm_dim < 0 || a.stat_groups < 0 ||
      (a.norm_dim > 0 && (a.stat_groups < 1 || !a.stat_in || (!a.rms && !a.wg) || (a.publish && !a.rms && !a.cen))))
    SS_FAIL(SS_EINVAL, "decode attention: incomplete normalisation arguments for raw q|k|v");
  if (a.rows_per_block < 1 || a.splits < 1 || (size_t)a.splits * a.rows_per_block < (size_t)a.Smax)
    SS_FAIL(SS_EINVAL, "decode attention: %d splits of %d rows do not cover %d rows", a.splits, a.rows_per_block, a.Smax);
  return SS_OK;
}

ss_status launch_decode_attn(int dtype, const DecodeAttnArgs &a, hipStream_t st) {
  SS_TRY(check_decode_attn(a));
  dim3 grid(a.B * a.Hs, a.splits);
#define SS_LAUNCH(KT, AT, DH)                                                                        \
  do {                                                                                               \
    if (a.norm_dim > 0) {  /* raw q|k|v: the kernel applies the normalisation */                      \
      if (a.waves == 16) SS_LAUNCH_KERNEL((decode_attn<KT, AT, DH, 16, true>), grid, dim3(1024), 0, st, a); \
      else if (a.waves == 8) SS_LAUNCH_KERNEL((decode_attn<KT, AT, DH, 8, true>), grid, dim3(512), 0, st, a); \
      else SS_LAUNCH_KERNEL((decode_attn<KT, AT, DH, 4, true>), grid, dim3(256), 0, st, a);          \
    } else if (a.waves == 16) SS_LAUNCH_KERNEL((decode_attn<KT, AT, DH, 16, false>), grid, dim3(1024), 0, st, a); \
    else if (a.waves == 8) SS_LAUNCH_KERNEL((decode_attn<KT, AT, DH, 8, false>), grid, dim3(512), 0, st, a); \
    else SS_LAUNCH_KERNEL((decode_attn<KT, AT, DH, 4, false>), grid, dim3(256), 0, st, a);           \
  } while (0)
  if (dtype == SS_DTYPE_BF16 && a.kv_dtype == SS_DTYPE_F16) {  // bf16 models: the output operand is halves
    if (a.Dh == 128) SS_LAUNCH(f16_t, f16_t, 128);
    else SS_LAUNCH(f16_t, f16_t, 64);
  } else if (dtype == SS_DTYPE_BF16 && a.kv_dtype == SS_DTYPE_BF16) {
    if (a.Dh == 128) SS_LAUNCH(bf16_t, f16_t, 128);
    else SS_LAUNCH(bf16_t, f16_t, 64);
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
// initial phase: rotate q (in place) and k, write K/V rows of all prompt positions.
// DH/8 threads per (token, head), each with four dims of both halves of the head (a rotation
// pairs dim e with e + DH/2); 256 threads per block.
// ---------------------------------------------------------------------------
template <typename T, int DH>
__global__ void __launch_bounds__(256) prefill_kv_write(PrefillAttnArgs a) {
  constexpr int HALF = DH / 2, TPP = HALF / 4, PPB = 256 / TPP;
  const int pair = blockIdx.x * PPB + threadIdx.x / TPP;
  if (pair >= a.B * a.S * a.Hs) return;
  const int t = pair / a.Hs, h = pair - t * a.Hs, e0 = (threadIdx.x % TPP) * 4;
  const int b = t / a.S, pos = t - b * a.S;
  const int HD = a.Hs * DH;
  float *row = a.qkv + (size_t)t * 3 * HD + h * DH;
  f32x4 qlo = *(const f32x4 *)(row + e0), qhi = *(const f32x4 *)(row + HALF + e0);
  f32x4 klo = *(const f32x4 *)(row + HD + e0), khi = *(const f32x4 *)(row + HD + HALF + e0);
  const f32x4 vlo = *(const f32x4 *)(row + 2 * HD + e0), vhi = *(const f32x4 *)(row + 2 * HD + HALF + e0);
  if (a.rope) {
    const float2 *tab = a.rope + (size_t)pos * HALF + e0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float2 cs = tab[i];
      float ql, qh, kl, kh;
      rope_rotate(qlo[i], qhi[i], cs, ql, qh);
      rope_rotate(klo[i], khi[i], cs, kl, kh);
      qlo[i] = ql, qhi[i] = qh, klo[i] = kl, khi[i] = kh;
    }
    *(f32x4 *)(row + e0) = qlo;
    *(f32x4 *)(row + HALF + e0) = qhi;
  }
  const size_t off = b * a.row_stride + h * a.head_stride + (size_t)pos * DH * sizeof(T);
  T *kc = (T *)(a.k_cache + off), *vc = (T *)(a.v_cache + off);
  store4_cache<T>(kc + e0, klo);
  store4_cache<T>(kc + HALF + e0, khi);
  store4_cache<T>(vc + e0, vlo);
  store4_cache<T>(vc + HALF + e0, vhi);
}

ss_status launch_prefill_kv_write(int dtype, const PrefillAttnArgs &a, hipStream_t st) {
  if (a.S < 1 || a.S > a.Smax || a.B < 1 || (a.Dh != 64 && a.Dh != 128)) SS_FAIL(SS_EINVAL, "prefill KV write: bad shape");
  const int pairs_per_block = 256 / (a.Dh / 8);
  dim3 grid(ceil_div(a.B * a.S * a.Hs, pairs_per_block));
#define SS_LAUNCH(KT, DH) hipLaunchKernelGGL((prefill_kv_write<KT, DH>), grid, dim3(256), 0, st, a)
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
      store_act<AT>(a.o_out, tok, h * DH + part * DP + e, HD / Elem<AT>::kFragK, acc[e] * inv);
  }
}

// ---------------------------------------------------------------------------
// causal attention of the initial phase on the matrix cores (half-precision cache).
//
// prefill_vt_write: this layer's value rows, transposed: vt[(b*Hs + h)][dim][pos], pos < s_pad
// (a multiple of 64), zeros past S, so that the P.V product finds the key index contiguous.
// grid = (B*Hs, s_pad/64); a tile of 64 positions x DH dims goes through LDS.
// ---------------------------------------------------------------------------
template <int DH>
__global__ void __launch_bounds__(256) prefill_vt_write(PrefillAttnArgs a) {
  __shared__ f16_t tile[64][DH + 2];
  const int tid = threadIdx.x, bh = blockIdx.x, p0 = blockIdx.y * 64;
  const int b = bh / a.Hs, h = bh - b * a.Hs;
  const char *vbase = a.v_cache + b * a.row_stride + h * a.head_stride;
  constexpr int RP = DH / 8;  // 16-byte pieces per row
  for (int p = tid; p < 64 * RP; p += 256) {
    const int row = p / RP, pc = p - row * RP;
    u32x4 raw = {0u, 0u, 0u, 0u};
    if (p0 + row < a.S) raw = *((const u32x4 *)(vbase + (size_t)(p0 + row) * DH * sizeof(f16_t)) + pc);
    f16_t v[8];
    __builtin_memcpy(v, &raw, 16);
#pragma unroll
    for (int e = 0; e < 8; ++e) tile[row][pc * 8 + e] = v[e];
  }
  __syncthreads();
  f16_t *out = (f16_t *)a.vt + (size_t)bh * DH * a.s_pad + p0;
  for (int p = tid; p < DH * 8; p += 256) {
    const int dim = p >> 3, pc = p & 7;
    f16_t v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = tile[pc * 8 + e][dim];
    u32x4 raw;
    __builtin_memcpy(&raw, v, 16);
    *(u32x4 *)(out + (size_t)dim * a.s_pad + pc * 8) = raw;
  }
}

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// grid = (B*Hs, ceil(S/64)); block = 4 waves, wave w owns queries 64*qt + 16*w .. + 15.
// Keys go 32 at a time through a double-buffered LDS tile in operand order.  Per 16 keys:
//   scores^T = K . Q^T   (16x16x32 products over the head dims): lane (g, r) gets the scores of keys
//                        4g .. 4g+3 against query r, so a query's softmax state lives in lane r of
//                        each of the four lane groups;
//   out^T   += V^T . P^T (one 16x16x32 product over the 32 keys of a tile): the lane's four probabilities of each
//                        of the tile's two subtiles are exactly its piece of the P operand, nothing is exchanged between lanes.
// Scores are kept in log2 units (the scale carries log2 e).  q and the probabilities enter the
// products as halves, keys and values at cache precision.
template <typename AT, int DH>
__global__ void __launch_bounds__(256) prefill_attn_mfma(PrefillAttnArgs a) {
  constexpr int TK = 32, KC = DH / 32, DT = DH / 16;
  __shared__ __align__(16) u32x4 lds_k[2][2][KC][64];  // [buffer][16-key subtile][32-dim block][lane]
  // [buffer][16-key subtile][16-dim tile][lane (g, r) at g * 16 + (r ^ 8 * (g >> 1))] + 16 entries between the subtiles: the
  // staging stores of a wave (16 dims x 4 key pieces) then fall on distinct banks, as the reads (one entry per lane) do anyway
  __shared__ __align__(16) uint2 lds_v[2][2][DT * 64 + 16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, g = lane >> 4;
  const int bh = blockIdx.x, qt = gridDim.y - 1 - blockIdx.y;  // the longest tiles start first
  const int b = bh / a.Hs, h = bh - b * a.Hs;
  const int HD = a.Hs * DH;
  const int q0 = qt * 64 + wave * 16, qi = q0 + r;
  const float sc = rsqrtf((float)DH) * 1.4426950408889634f;
  f16x8 qf[KC];
  {
    const float *qrow = a.qkv + ((size_t)(b * a.S + min(qi, a.S - 1))) * 3 * HD + h * DH;
#pragma unroll
    for (int c = 0; c < KC; ++c)
#pragma unroll
      for (int e = 0; e < 8; ++e) qf[c][e] = (f16_t)(qrow[c * 32 + g * 8 + e] * sc);
  }
  f32x4 acc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m = -1e30f, l = 0.f;
  const char *kbase = a.k_cache + b * a.row_stride + h * a.head_stride;
  const f16_t *vt = (const f16_t *)a.vt + (size_t)bh * DH * a.s_pad;
  const int last_key = min(a.S, (qt + 1) * 64);
  const int n_tiles = (last_key + TK - 1) / TK;

  // staging: 32 keys x DH halves of K = 4*DH pieces of 16 bytes, and as many of V^T (DH dims x 32 keys)
  constexpr int NP = 4 * DH / 256;  // pieces per thread and operand
  u32x4 kreg[NP], vreg[NP];
  auto fetch = [&](int t) {
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int p = tid + 256 * i;
      // a wave takes one whole LDS fragment (16 keys x 4 pieces): lane l holds key l & 15, piece l >> 4 of it
      const int key = (p >> 6) / KC * 16 + (p & 15), pc = (p >> 6) % KC * 4 + ((p >> 4) & 3);
      const int kr = min(t * TK + key, a.S - 1);  // clamped: masked below
      kreg[i] = *((const u32x4 *)(kbase + (size_t)kr * DH * sizeof(f16_t)) + pc);
      const int dim = p >> 2, kp = p & 3;         // 8 keys of one dim (inside s_pad, zeros past S)
      vreg[i] = *(const u32x4 *)(vt + (size_t)dim * a.s_pad + t * TK + kp * 8);
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int p = tid + 256 * i;
      lds_k[buf][(p >> 6) / KC][(p >> 6) % KC][p & 63] = kreg[i];  // consecutive lanes, consecutive 16 bytes: no bank conflicts
      const int dim = p >> 2, kp = p & 3;
      uint2 *dst = &lds_v[buf][kp >> 1][(dim >> 4) * 64 + ((kp & 1) * 2) * 16 + ((dim & 15) ^ ((kp & 1) * 8))];
      dst[0] = make_uint2(vreg[i][0], vreg[i][1]);    // keys 8*(kp&1) .. + 3 of the subtile
      dst[16] = make_uint2(vreg[i][2], vreg[i][3]);   // the next four: lane group + 1
    }
  };
  fetch(0);
  stash(0);
  __syncthreads();
  for (int t = 0; t < n_tiles; ++t) {
    const int buf = t & 1;
    const bool more = t + 1 < n_tiles;
    if (more) fetch(t + 1);
    // The tile's two 16-key subtiles take one softmax step together (one exchange of maxima, one rescaling of the sums),
    // and their probabilities are the two halves of the P operand of one 16x16x32 product per 16 dims: the product's k
    // index runs over (subtile 0, keys 4g .. 4g+3), (subtile 1, keys 4g .. 4g+3) in lane group g, for P as for V^T.
    const int key0 = t * TK;
    if (!(key0 > q0 + 15 || key0 >= a.S)) {  // else nothing of this tile is visible to the wave's queries
      const bool vis1 = !(key0 + 16 > q0 + 15 || key0 + 16 >= a.S);
      f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
      for (int c = 0; c < KC; ++c)
        s0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, lds_k[buf][0][c][lane]), qf[c], s0, 0, 0, 0);
      if (vis1) {
        s1 = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < KC; ++c)
          s1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, lds_k[buf][1][c][lane]), qf[c], s1, 0, 0, 0);
      }
      float mx = -INFINITY;
      if (key0 + 31 <= q0 && key0 + 32 <= a.S) {  // every key of the tile is visible to every query of the wave (wave-uniform)
#pragma unroll
        for (int i = 0; i < 4; ++i) mx = fmaxf(mx, fmaxf(s0[i], s1[i]));
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int ka = key0 + g * 4 + i, kb = ka + 16;
          s0[i] = (ka <= qi && ka < a.S) ? s0[i] : -INFINITY;
          s1[i] = (kb <= qi && kb < a.S) ? s1[i] : -INFINITY;
          mx = fmaxf(mx, fmaxf(s0[i], s1[i]));
        }
      }
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float mn = fmaxf(m, mx);
      const float alpha = __builtin_amdgcn_exp2f(m - mn);
      f16x8 pf;
      float ps = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float p0 = __builtin_amdgcn_exp2f(s0[i] - mn), p1 = __builtin_amdgcn_exp2f(s1[i] - mn);
        ps += p0 + p1;
        pf[i] = (f16_t)p0, pf[4 + i] = (f16_t)p1;
      }
      l = l * alpha + ps;
      m = mn;
      const int vl = lane ^ ((lane >> 5) * 8);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        acc[dt] *= alpha;
        const uint2 va = lds_v[buf][0][dt * 64 + vl], vb = lds_v[buf][1][dt * 64 + vl];
        const u32x4 v8 = {va.x, va.y, vb.x, vb.y};
        acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, v8), pf, acc[dt], 0, 0, 0);
      }
    }
    if (more) stash(buf ^ 1);  // last read in the previous iteration, before its barrier
    __syncthreads();
  }
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  if (qi < a.S) {
    const float inv = 1.0f / l;
    const int tok = b * a.S + qi;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const float v[4] = {acc[dt][0] * inv, acc[dt][1] * inv, acc[dt][2] * inv, acc[dt][3] * inv};
      store4_frag<AT, false>(a.o_out, tok, h * DH + dt * 16 + g * 4, HD / Elem<AT>::kFragK, v);
    }
  }
}

ss_status launch_prefill_attn(int dtype, const PrefillAttnArgs &a, hipStream_t st) {
  if (a.S < 1 || a.S > a.Smax || a.B < 1 || (a.Dh != 64 && a.Dh != 128)) SS_FAIL(SS_EINVAL, "prefill attention: bad shape");
  dim3 grid(a.B * a.Hs, ceil_div(a.S, 64));
#define SS_LAUNCH(KT, AT, DH) hipLaunchKernelGGL((prefill_attn<KT, AT, DH>), grid, dim3(256), 0, st, a)
  if (dtype == SS_DTYPE_BF16 && a.kv_dtype == SS_DTYPE_F16) {  // the default cache type: matrix cores
    if (!a.vt || a.s_pad < a.S || a.s_pad % 64) SS_FAIL(SS_EINVAL, "prefill attention: no room for the transposed values");
    dim3 tgrid(a.B * a.Hs, a.s_pad / 64);
    if (a.Dh == 128) {
      hipLaunchKernelGGL((prefill_vt_write<128>), tgrid, dim3(256), 0, st, a);
      hipLaunchKernelGGL((prefill_attn_mfma<f16_t, 128>), grid, dim3(256), 0, st, a);
    } else {
      hipLaunchKernelGGL((prefill_vt_write<64>), tgrid, dim3(256), 0, st, a);
      hipLaunchKernelGGL((prefill_attn_mfma<f16_t, 64>), grid, dim3(256), 0, st, a);
    }
  } else if (dtype == SS_DTYPE_BF16 && a.kv_dtype == SS_DTYPE_BF16) {  // output: single half-precision fragments
    if (a.Dh == 128) SS_LAUNCH(bf16_t, f16_t, 128);
    else SS_LAUNCH(bf16_t, f16_t, 64);
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
