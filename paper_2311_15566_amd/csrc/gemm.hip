// GEMM kernels on the matrix cores: the skinny (decode) weight-streaming GEMM with fused
// prologues/epilogues, and the tiled prefill GEMM.
#include "kernels.h"

#include <limits.h>
#include <math.h>
#include <stdlib.h>

#include <algorithm>

namespace ss {

// ---------------------------------------------------------------------------
// one 16 x 16 x FragK product per call: D[n][b] += sum_k W[n][k] * A[b][k]
// lane l returns D[(l>>4)*4 + i][l & 15], i = 0..3
// ---------------------------------------------------------------------------
template <typename T> struct Mma;
template <> struct Mma<bf16_t> {
  static __device__ __forceinline__ f32x4 mma(u32x4 w, u32x4 a, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w), __builtin_bit_cast(bf16x8, a), c, 0,
                                                   0, 0);
  }
};
template <> struct Mma<float> {
  static __device__ __forceinline__ f32x4 mma(u32x4 w, u32x4 a, f32x4 c) {
    f32x4 wf = __builtin_bit_cast(f32x4, w), af = __builtin_bit_cast(f32x4, a);
#pragma unroll
    for (int j = 0; j < 4; ++j) c = __builtin_amdgcn_mfma_f32_16x16x4f32(wf[j], af[j], c, 0, 0, 0);
    return c;
  }
};

__device__ __forceinline__ float act_apply(int kind, float h) {
  if (kind == SS_ACT_GELU_TANH) return 0.5f * h * (1.0f + tanhf(0.7978845608028654f * (h + 0.044715f * h * h * h)));
  return fmaxf(h, 0.0f);  // SS_ACT_RELU
}
__device__ __forceinline__ float silu_f(float g) { return g / (1.0f + __expf(-g)); }

template <typename T>
__device__ __forceinline__ void store4_frag(void *base, int row, int k, int k_blocks, int parts, float v0, float v1,
                                            float v2, float v3) {
  // k is a multiple of 4: the four values are contiguous within a part
  const float v[4] = {v0, v1, v2, v3};
  T *hi = (T *)base + frag_offset_parts<T>(row, k, k_blocks, parts, 0);
#pragma unroll
  for (int i = 0; i < 4; ++i) hi[i] = Elem<T>::from_f32(v[i]);
  if (parts > 1) {
    T *lo = (T *)base + frag_offset_parts<T>(row, k, k_blocks, parts, 1);
#pragma unroll
    for (int i = 0; i < 4; ++i) lo[i] = Elem<T>::from_f32(v[i] - Elem<T>::to_f32(hi[i]));
  }
}

// ---------------------------------------------------------------------------
// skinny GEMM.  grid = (groups of 4 wave tasks, K splits); block = 4 waves.
// A wave owns one 16-row weight tile (SwiGLU: a gate/up tile pair) over the block's K range
// and streams it in register batches of U fragments, two batches in flight (the first is
// requested before the block stages its activations).  The activations of the K range are
// staged once per block in LDS, normalised on the way in for the norm prologue.
// ---------------------------------------------------------------------------
template <typename T, int NB, int NW, int PRO, int EPI>
__global__ void __launch_bounds__(256) skinny_gemm(SkinnyArgs a) {
  constexpr int PL = Elem<T>::kPerLane, FK = Elem<T>::kFragK, AP = Elem<T>::kParts;
  constexpr int U = NW == 1 ? 8 : 4;
  extern __shared__ __align__(16) char smem[];  // [NB][lds_chunk][AP] fragments of the activations
  __shared__ float red_f[4][32][2];
  __shared__ int red_i[4][32];
  __shared__ int s_flag;
  u32x4 *lds = (u32x4 *)smem;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int group = blockIdx.x, sp = blockIdx.y;
  const int task = group * 4 + wave;
  const bool live = task < a.tasks;
  const int kb0 = sp * a.kb_per_split;
  const int nk = min(a.kb_per_split, a.k_blocks - kb0);  // fragments along K for this block
  const int K = a.k_blocks * FK;

  f32x4 acc[NB][NW];
#pragma unroll
  for (int t = 0; t < NB; ++t)
#pragma unroll
    for (int j = 0; j < NW; ++j) acc[t][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  const u32x4 *wbase = (const u32x4 *)a.w + ((size_t)task * NW * a.k_blocks + kb0) * 64 + lane;
  auto load_batch = [&](u32x4(&buf)[NW][U], int kb) {
#pragma unroll
    for (int j = 0; j < NW; ++j)
#pragma unroll
      for (int u = 0; u < U; ++u)
        buf[j][u] = (live && kb + u < nk) ? __builtin_nontemporal_load(wbase + ((size_t)j * a.k_blocks + kb + u) * 64)
                                          : u32x4{0u, 0u, 0u, 0u};
  };
  auto compute = [&](u32x4(&buf)[NW][U], int kb, int nkb) {  // kb relative to the staged chunk
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (kb + u < nkb) {
#pragma unroll
        for (int t = 0; t < NB; ++t)
#pragma unroll
          for (int part = 0; part < AP; ++part) {
            const u32x4 af = lds[((t * a.lds_chunk + kb + u) * AP + part) * 64 + lane];
#pragma unroll
            for (int j = 0; j < NW; ++j) acc[t][j] = Mma<T>::mma(buf[j][u], af, acc[t][j]);
          }
      }
  };

  u32x4 cur[NW][U], nxt[NW][U];
  load_batch(cur, 0);

  for (int c0 = 0; c0 < nk; c0 += a.lds_chunk) {  // lds_chunk is a multiple of 2U when it is < nk
    const int nkb = min(a.lds_chunk, nk - c0);
    if (c0) __syncthreads();
    if (PRO == PRO_ACT) {
      const u32x4 *src = (const u32x4 *)a.act;
      const int per = nkb * AP * 64;
      for (int i = tid; i < NB * per; i += 256) {
        const int t = i / per, r = i - t * per;
        lds[t * a.lds_chunk * AP * 64 + r] = src[((size_t)t * a.k_blocks + kb0 + c0) * AP * 64 + r];
      }
    } else {
      const int ppr = nkb * 4;  // 16-byte pieces per row in this chunk
      for (int i = tid; i < a.B * ppr; i += 256) {
        const int row = i / ppr, p = i - row * ppr;
        const int k0 = (kb0 + c0) * FK + p * PL;
        const float mean = a.stats[row * 2], rstd = a.stats[row * 2 + 1];
        const f32x4 *xp = (const f32x4 *)(a.x + (size_t)row * K + k0);
        const f32x4 *gp = (const f32x4 *)(a.gamma + k0);
        const f32x4 *bp = (const f32x4 *)(a.beta + k0);
        T v[AP][PL];
#pragma unroll
        for (int q = 0; q < PL / 4; ++q) {
          const f32x4 xv = xp[q], gv = gp[q];
          f32x4 y = (xv - mean) * rstd * gv;
          if (a.beta) y += bp[q];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v[0][q * 4 + e] = Elem<T>::from_f32(y[e]);
            if (AP > 1) v[AP - 1][q * 4 + e] = Elem<T>::from_f32(y[e] - Elem<T>::to_f32(v[0][q * 4 + e]));
          }
        }
#pragma unroll
        for (int part = 0; part < AP; ++part) {
          u32x4 packed;
          __builtin_memcpy(&packed, v[part], 16);
          lds[(((row >> 4) * a.lds_chunk + (p >> 2)) * AP + part) * 64 + (p & 3) * 16 + (row & 15)] = packed;
        }
      }
    }
    __syncthreads();
    for (int kb = 0; kb < nkb; kb += 2 * U) {
      load_batch(nxt, c0 + kb + U);
      compute(cur, kb, nkb);
      load_batch(cur, c0 + kb + 2 * U);
      compute(nxt, kb + U, nkb);
    }
  }

  const int q4 = (lane >> 4) * 4;  // this lane's four consecutive output features within the tile
  const int bl = lane & 15;        // this lane's batch row within the tile

  // ---- split-K: the last block to arrive for this group sums the partials in split order ----
  if (a.split > 1) {
    const size_t npad = (size_t)a.tasks * NW * 16;
    if (live) {
#pragma unroll
      for (int t = 0; t < NB; ++t)
        if (t * 16 + bl < a.B) {
#pragma unroll
          for (int j = 0; j < NW; ++j) {
            float *p = a.splitk + ((size_t)sp * NB * 16 + t * 16 + bl) * npad + (size_t)(task * NW + j) * 16 + q4;
#pragma unroll
            for (int i = 0; i < 4; ++i) st_dev(p + i, acc[t][j][i]);
          }
        }
    }
    if (!arrive_last(&a.counters[group], a.split, &s_flag)) return;
    if (live) {
#pragma unroll
      for (int t = 0; t < NB; ++t)
        if (t * 16 + bl < a.B) {
#pragma unroll
          for (int j = 0; j < NW; ++j) {
            // partials are summed in split order; loads are issued four splits at a time
            f32x4 sum = f32x4{0.f, 0.f, 0.f, 0.f};
            const float *p0 = a.splitk + ((size_t)t * 16 + bl) * npad + (size_t)(task * NW + j) * 16 + q4;
            const size_t sstride = (size_t)NB * 16 * npad;
            int s2 = 0;
            for (; s2 + 4 <= a.split; s2 += 4) {
              float v[4][4];
#pragma unroll
              for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int i = 0; i < 4; ++i) v[r][i] = ld_dev(p0 + (size_t)(s2 + r) * sstride + i);
#pragma unroll
              for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int i = 0; i < 4; ++i) sum[i] += v[r][i];
            }
            for (; s2 < a.split; ++s2)
#pragma unroll
              for (int i = 0; i < 4; ++i) sum[i] += ld_dev(p0 + (size_t)s2 * sstride + i);
            acc[t][j] = sum;
          }
        }
    }
  }

  const int n0 = task * 16 + q4;
  if (EPI == EPI_F32) {
    if (live) {
#pragma unroll
      for (int t = 0; t < NB; ++t) {
        const int b = t * 16 + bl;
        if (b < a.B) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int n = n0 + i;
            if (n < a.N) a.out_f32[(size_t)b * a.ld_out + n] = acc[t][0][i] + (a.bias ? a.bias[n] : 0.f);
          }
        }
      }
    }
    return;
  }
  if (EPI == EPI_ACT || EPI == EPI_SWIGLU) {
    if (live) {
#pragma unroll
      for (int t = 0; t < NB; ++t) {
        const int b = t * 16 + bl;
        if (b < a.B && n0 < a.N) {
          float u[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            if (EPI == EPI_SWIGLU) {
              u[i] = silu_f(acc[t][0][i]) * acc[t][NW - 1][i];
            } else {
              u[i] = act_apply(a.act_kind, acc[t][0][i] + (a.bias ? a.bias[n0 + i] : 0.f));
            }
          }
          store4_frag<T>(a.act_out, b, n0, a.out_k_blocks, AP, u[0], u[1], u[2], u[3]);
        }
      }
    }
    return;
  }
  if (EPI == EPI_RESID) {
    float s1[NB], s2[NB];
#pragma unroll
    for (int t = 0; t < NB; ++t) {
      s1[t] = 0.f, s2[t] = 0.f;
      const int b = t * 16 + bl;
      if (live && b < a.B) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int n = n0 + i;
          if (n < a.N) {
            float *xp = a.x_resid + (size_t)b * a.N + n;
            float v = *xp + acc[t][0][i] + (a.bias ? a.bias[n] : 0.f);
            *xp = v;
            s1[t] += v;
            s2[t] += v * v;
          }
        }
      }
      s1[t] += __shfl_xor(s1[t], 16);
      s2[t] += __shfl_xor(s2[t], 16);
      s1[t] += __shfl_xor(s1[t], 32);
      s2[t] += __shfl_xor(s2[t], 32);
      if (lane < 16) red_f[wave][t * 16 + lane][0] = s1[t], red_f[wave][t * 16 + lane][1] = s2[t];
    }
    __syncthreads();
    if (tid < NB * 16) {
      float p1 = 0.f, p2 = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) p1 += red_f[w][tid][0], p2 += red_f[w][tid][1];
      st_dev(&a.stat_part[((size_t)group * 32 + tid) * 2 + 0], p1);
      st_dev(&a.stat_part[((size_t)group * 32 + tid) * 2 + 1], p2);
    }
    if (!arrive_last(&a.counters[gridDim.x], (int)gridDim.x, &s_flag)) return;
    {
      // thread (slice = tid / 32, b = tid % 32) sums groups slice, slice + 8, ... in order; the 8
      // slices are then added in order, so the result does not depend on scheduling
      const int b = tid & 31, slice = tid >> 5;
      float t1 = 0.f, t2 = 0.f;
      if (b < a.B) {
#pragma unroll 4
        for (int g = slice; g < (int)gridDim.x; g += 8) {
          t1 += ld_dev(&a.stat_part[((size_t)g * 32 + b) * 2 + 0]);
          t2 += ld_dev(&a.stat_part[((size_t)g * 32 + b) * 2 + 1]);
        }
      }
      __shared__ float fin[8][32][2];
      fin[slice][b][0] = t1, fin[slice][b][1] = t2;
      __syncthreads();
      if (tid < a.B) {
        float u1 = 0.f, u2 = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) u1 += fin[q][tid][0], u2 += fin[q][tid][1];
        const float inv = 1.0f / (float)a.N;
        float mean = u1 * inv, ms = u2 * inv;
        float rstd;
        if (a.rms) {
          rstd = rsqrtf(ms + a.eps);
          mean = 0.f;
        } else {
          rstd = rsqrtf(fmaxf(ms - mean * mean, 0.f) + a.eps);
        }
        a.stats_out[tid * 2 + 0] = mean;
        a.stats_out[tid * 2 + 1] = rstd;
      }
    }
    return;
  }
  if (EPI == EPI_LOGITS) {
#pragma unroll
    for (int t = 0; t < NB; ++t) {
      float bv = -INFINITY;
      int bi = INT_MAX;
      const int b = t * 16 + bl;
      if (live) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int n = n0 + i;
          if (n < a.N) {
            const float v = acc[t][0][i];
            if (a.out_f32 && b < a.B) a.out_f32[(size_t)b * a.ld_out + n] = v;
            if (v > bv) bv = v, bi = n;
          }
        }
      }
#pragma unroll
      for (int off = 16; off <= 32; off <<= 1) {
        float ov = __shfl_xor(bv, off);
        int oi = __shfl_xor(bi, off);
        if (ov > bv || (ov == bv && oi < bi)) bv = ov, bi = oi;
      }
      if (lane < 16) red_f[wave][t * 16 + lane][0] = bv, red_i[wave][t * 16 + lane] = bi;
    }
    __syncthreads();
    if (tid < NB * 16) {
      float bv = red_f[0][tid][0];
      int bi = red_i[0][tid];
#pragma unroll
      for (int w = 1; w < 4; ++w) {
        float ov = red_f[w][tid][0];
        int oi = red_i[w][tid];
        if (ov > bv || (ov == bv && oi < bi)) bv = ov, bi = oi;
      }
      st_dev(&a.am_val[(size_t)group * 32 + tid], bv);
      st_dev(&a.am_idx[(size_t)group * 32 + tid], bi);
    }
    if (!arrive_last(&a.counters[gridDim.x], (int)gridDim.x, &s_flag)) return;
    {
      // thread (slice = tid / 32, b = tid % 32) scans groups slice, slice + 8, ...; ties go to the
      // lowest index whatever the order, so the merge over slices is order-independent
      const int b = tid & 31, slice = tid >> 5;
      float bv = -INFINITY;
      int bi = INT_MAX;
      if (b < a.B) {
#pragma unroll 4
        for (int g = slice; g < (int)gridDim.x; g += 8) {
          const float ov = ld_dev(&a.am_val[(size_t)g * 32 + b]);
          const int oi = ld_dev(&a.am_idx[(size_t)g * 32 + b]);
          if (ov > bv || (ov == bv && oi < bi)) bv = ov, bi = oi;
        }
      }
      __shared__ float fin_v[8][32];
      __shared__ int fin_i[8][32];
      fin_v[slice][b] = bv, fin_i[slice][b] = bi;
      __syncthreads();
      if (tid < a.B) {
        bv = fin_v[0][tid], bi = fin_i[0][tid];
#pragma unroll
        for (int q = 1; q < 8; ++q) {
          const float ov = fin_v[q][tid];
          const int oi = fin_i[q][tid];
          if (ov > bv || (ov == bv && oi < bi)) bv = ov, bi = oi;
        }
        if (a.next_tokens) a.next_tokens[tid] = bi;
        // token-level commit: the last action of the step
        for (int q = 0; q < a.n_lens; ++q) a.lens[q][tid] += a.commit_inc;
      }
    }
    return;
  }
}

static int env_int(const char *name, int dflt) {
  const char *v = getenv(name);
  return v && *v ? atoi(v) : dflt;
}

void plan_skinny(SkinnyArgs *a, int esz, size_t splitk_bytes, int nw) {
  a->nb = a->B <= 16 ? 1 : 2;
  const int groups = ceil_div(a->tasks, 4);
  static const int target_blocks = env_int("SS_SKINNY_BLOCKS", 512);  // about 2 blocks per compute unit
  static const int lds_kb = env_int("SS_SKINNY_LDS_KB", 64);
  const int parts = esz == 2 ? 2 : 1;                                   // bf16 activations are hi/lo pairs
  const int max_chunk = std::max(16, lds_kb / (a->nb * parts) / 16 * 16);  // k blocks staged at a time, multiple of 16
  int split = std::max(1, std::min(target_blocks / std::max(groups, 1), a->k_blocks / 4));
  const size_t per_split = (size_t)a->nb * 16 * a->tasks * nw * 16 * 4;
  while (split > 1 && per_split * split > splitk_bytes) --split;
  a->kb_per_split = ceil_div(a->k_blocks, split);
  a->split = ceil_div(a->k_blocks, a->kb_per_split);
  a->lds_chunk = a->kb_per_split <= max_chunk ? a->kb_per_split : max_chunk;
}

template <typename T, int NB>
static void launch_skinny_t(int pro, int epi, const SkinnyArgs &a, dim3 grid, size_t lds, hipStream_t st) {
#define SS_LAUNCH(NW, PRO, EPI) hipLaunchKernelGGL((skinny_gemm<T, NB, NW, PRO, EPI>), grid, dim3(256), lds, st, a)
  if (pro == PRO_NORM && epi == EPI_F32) SS_LAUNCH(1, PRO_NORM, EPI_F32);
  else if (pro == PRO_NORM && epi == EPI_LOGITS) SS_LAUNCH(1, PRO_NORM, EPI_LOGITS);
  else if (pro == PRO_NORM && epi == EPI_ACT) SS_LAUNCH(1, PRO_NORM, EPI_ACT);
  else if (pro == PRO_NORM && epi == EPI_SWIGLU) SS_LAUNCH(2, PRO_NORM, EPI_SWIGLU);
  else if (pro == PRO_ACT && epi == EPI_RESID) SS_LAUNCH(1, PRO_ACT, EPI_RESID);
#undef SS_LAUNCH
}

ss_status launch_skinny(int dtype, int pro, int epi, const SkinnyArgs &a, hipStream_t st) {
  const bool ok_combo = (pro == PRO_NORM && (epi == EPI_F32 || epi == EPI_LOGITS || epi == EPI_ACT || epi == EPI_SWIGLU)) ||
                        (pro == PRO_ACT && epi == EPI_RESID);
  if (!ok_combo) SS_FAIL(SS_EINVAL, "skinny GEMM: unsupported prologue/epilogue pair %d/%d", pro, epi);
  if (a.B < 1 || a.B > 32 || a.nb != (a.B <= 16 ? 1 : 2)) SS_FAIL(SS_EINVAL, "skinny GEMM: batch %d / tiles %d", a.B, a.nb);
  if (a.tasks < 1 || a.k_blocks < 1 || a.split < 1 || a.kb_per_split < 1 || a.lds_chunk < 1 ||
      (size_t)a.split * a.kb_per_split < (size_t)a.k_blocks || a.lds_chunk * a.nb * (dtype == SS_DTYPE_BF16 ? 2 : 1) > 64 ||
      (a.lds_chunk < a.kb_per_split && a.lds_chunk % 16))
    SS_FAIL(SS_EINVAL, "skinny GEMM: inconsistent plan");
  const int groups = ceil_div(a.tasks, 4);
  dim3 grid(groups, a.split);
  size_t lds = (size_t)a.nb * a.lds_chunk * (dtype == SS_DTYPE_BF16 ? 2 : 1) * 1024;
  if (dtype == SS_DTYPE_BF16) {
    if (a.nb == 1) launch_skinny_t<bf16_t, 1>(pro, epi, a, grid, lds, st);
    else launch_skinny_t<bf16_t, 2>(pro, epi, a, grid, lds, st);
  } else {
    if (a.nb == 1) launch_skinny_t<float, 1>(pro, epi, a, grid, lds, st);
    else launch_skinny_t<float, 2>(pro, epi, a, grid, lds, st);
  }
  SS_HIP(hipGetLastError());
  return SS_OK;
}

// ---------------------------------------------------------------------------
// tiled prefill GEMM: block = 128 output features x 128 tokens, 4 waves of 64 x 64,
// K advanced two fragments at a time through LDS with register prefetch of the next stage.
// ---------------------------------------------------------------------------
template <typename T, int EPI, int AP>
__global__ void __launch_bounds__(256) tile_gemm(TileGemmArgs a) {
  constexpr int KS = 2;  // k fragments per stage
  __shared__ __align__(16) u32x4 lds_w[KS][8][64];
  __shared__ __align__(16) u32x4 lds_a[KS][8][AP][64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 1, wc = wave & 1;
  const int rt0 = blockIdx.x * 8;   // first weight row tile
  const int tt0 = blockIdx.y * 8;   // first token tile
  const u32x4 *W = (const u32x4 *)a.w;
  const u32x4 *A = (const u32x4 *)a.act;

  f32x4 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // per stage each thread moves 4 weight pieces and 4*AP activation pieces:
  // piece p = tid + 256*r -> (ks = p / 512, tile = (p / 64) % 8, ln = p % 64)
  u32x4 pw[4], pa[4][AP];
  auto fetch = [&](int kb) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int p = tid + 256 * r;
      const int ks = p >> 9, tile = (p >> 6) & 7, ln = p & 63;
      const int k = kb + ks;
      const bool kok = k < a.k_blocks;
      pw[r] = (kok && rt0 + tile < a.row_tiles) ? W[((size_t)(rt0 + tile) * a.k_blocks + k) * 64 + ln]
                                               : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
      for (int part = 0; part < AP; ++part)
        pa[r][part] = kok ? A[(((size_t)(tt0 + tile) * a.k_blocks + k) * AP + part) * 64 + ln] : u32x4{0u, 0u, 0u, 0u};
    }
  };
  fetch(0);
  for (int kb = 0; kb < a.k_blocks; kb += KS) {
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int p = tid + 256 * r;
      const int ks = p >> 9, tile = (p >> 6) & 7, ln = p & 63;
      lds_w[ks][tile][ln] = pw[r];
#pragma unroll
      for (int part = 0; part < AP; ++part) lds_a[ks][tile][part][ln] = pa[r][part];
    }
    __syncthreads();
    if (kb + KS < a.k_blocks) fetch(kb + KS);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      u32x4 wf[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) wf[i] = lds_w[ks][wr * 4 + i][lane];
#pragma unroll
      for (int part = 0; part < AP; ++part) {
        u32x4 af[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) af[j] = lds_a[ks][wc * 4 + j][part][lane];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = Mma<T>::mma(wf[i], af[j], acc[i][j]);
      }
    }
  }

  const int q4 = (lane >> 4) * 4, tl = lane & 15;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int tok = (tt0 + wc * 4 + j) * 16 + tl;
    if (EPI == EPI_SWIGLU) {
#pragma unroll
      for (int i = 0; i < 4; i += 2) {
        const int rt = rt0 + wr * 4 + i;  // gate tile; rt + 1 is the matching up tile
        const int n0 = (rt >> 1) * 16 + q4;
        if (rt + 1 < a.row_tiles && n0 < a.N) {
          float u[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) u[e] = silu_f(acc[i][j][e]) * acc[i + 1][j][e];
          store4_frag<T>(a.act_out, tok, n0, a.out_k_blocks, a.out_parts, u[0], u[1], u[2], u[3]);
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int rt = rt0 + wr * 4 + i;
        const int n0 = rt * 16 + q4;
        if (rt < a.row_tiles && n0 < a.N) {
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = acc[i][j][e] + (a.bias ? a.bias[n0 + e] : 0.f);
          if (EPI == EPI_F32) {
            *(f32x4 *)(a.out_f32 + (size_t)tok * a.ld_out + n0) = f32x4{v[0], v[1], v[2], v[3]};
          } else if (EPI == EPI_RESID) {
            f32x4 *xp = (f32x4 *)(a.x_resid + (size_t)tok * a.N + n0);
            f32x4 x = *xp;
            *xp = f32x4{x[0] + v[0], x[1] + v[1], x[2] + v[2], x[3] + v[3]};
          } else {  // EPI_ACT
            store4_frag<T>(a.act_out, tok, n0, a.out_k_blocks, a.out_parts, act_apply(a.act_kind, v[0]),
                           act_apply(a.act_kind, v[1]), act_apply(a.act_kind, v[2]), act_apply(a.act_kind, v[3]));
          }
        }
      }
    }
  }
}

ss_status launch_tile_gemm(int dtype, int epi, const TileGemmArgs &a, hipStream_t st) {
  if (a.T < 128 || a.T % 128) SS_FAIL(SS_EINVAL, "prefill GEMM: token count %d is not a multiple of 128", a.T);
  if (a.row_tiles < 1 || a.k_blocks < 1 || a.N % 4) SS_FAIL(SS_EINVAL, "prefill GEMM: bad shape");
  if ((epi == EPI_F32 && (a.ld_out % 4)) || epi == EPI_LOGITS) SS_FAIL(SS_EINVAL, "prefill GEMM: bad epilogue");
  if (a.act_parts != 1 && !(a.act_parts == 2 && dtype == SS_DTYPE_BF16)) SS_FAIL(SS_EINVAL, "prefill GEMM: bad act_parts");
  if ((epi == EPI_ACT || epi == EPI_SWIGLU) && a.out_parts != 1 && !(a.out_parts == 2 && dtype == SS_DTYPE_BF16))
    SS_FAIL(SS_EINVAL, "prefill GEMM: bad out_parts");
  dim3 grid(ceil_div(a.row_tiles, 8), a.T / 128);
#define SS_LAUNCH(TT, EPI, AP) hipLaunchKernelGGL((tile_gemm<TT, EPI, AP>), grid, dim3(256), 0, st, a)
  if (dtype == SS_DTYPE_BF16 && a.act_parts == 2) {
    if (epi == EPI_F32) SS_LAUNCH(bf16_t, EPI_F32, 2);
    else if (epi == EPI_RESID) SS_LAUNCH(bf16_t, EPI_RESID, 2);
    else if (epi == EPI_ACT) SS_LAUNCH(bf16_t, EPI_ACT, 2);
    else SS_LAUNCH(bf16_t, EPI_SWIGLU, 2);
  } else if (dtype == SS_DTYPE_BF16) {
    if (epi == EPI_F32) SS_LAUNCH(bf16_t, EPI_F32, 1);
    else if (epi == EPI_RESID) SS_LAUNCH(bf16_t, EPI_RESID, 1);
    else if (epi == EPI_ACT) SS_LAUNCH(bf16_t, EPI_ACT, 1);
    else SS_LAUNCH(bf16_t, EPI_SWIGLU, 1);
  } else {
    if (epi == EPI_F32) SS_LAUNCH(float, EPI_F32, 1);
    else if (epi == EPI_RESID) SS_LAUNCH(float, EPI_RESID, 1);
    else if (epi == EPI_ACT) SS_LAUNCH(float, EPI_ACT, 1);
    else SS_LAUNCH(float, EPI_SWIGLU, 1);
  }
#undef SS_LAUNCH
  SS_HIP(hipGetLastError());
  return SS_OK;
}

}  // namespace ss
