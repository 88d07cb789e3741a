// One block's share of the skinny (decode) GEMM, as a device function: the stand-alone kernel
// and the persistent decode-step kernel both call it.
#pragma once
#include <limits.h>
#include <math.h>

#include "kernels.h"
#include "mma.h"

namespace ss {

// small static LDS scratch of a skinny-GEMM block (cross-wave reductions, arrival flag)
struct SkinnyShared {
  float red_f[4][32][2];
  int red_i[4][32];
  float fin_f[8][32][2];
  int fin_i[8][32];
  int flag;
};

// Block (group, sp) of a grid of (ngroups, a.split) blocks of 4 waves.
// A wave owns one 16-row weight tile (SwiGLU: a gate/up tile pair) over the block's K range and
// streams it in register batches of U fragments, two batches in flight (the first is requested
// before the block stages its activations).  The activations of the K range are staged once
// per block in LDS, normalised on the way in for the norm prologue.
// lds: dynamic shared memory, a.nb * a.lds_chunk * parts KiB.
template <typename T, int NB, int NW, int PRO, int EPI>
__device__ __forceinline__ void skinny_block(const SkinnyArgs &a, const int group, const int sp, const int ngroups,
                                             u32x4 *lds, SkinnyShared &sh) {
  constexpr int PL = Elem<T>::kPerLane, FK = Elem<T>::kFragK, AP = Elem<T>::kParts;
  constexpr int U = NW == 1 ? 8 : 4;
  auto &red_f = sh.red_f;
  auto &red_i = sh.red_i;
  auto &fin_f = sh.fin_f;
  auto &fin_i = sh.fin_i;
  int &s_flag = sh.flag;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
    __syncthreads();  // the previous chunk (or the previous user of the LDS) is done
    if (PRO == PRO_ACT) {
      // operand-order activations [NB][k_blocks][AP][64 lanes]; lanes of dead batch rows are skipped
      const u32x4 *src = (const u32x4 *)a.act;
      const int per = nkb * AP * 64;
      for (int i = tid; i < NB * per; i += 256) {
        const int t = i / per, r = i - t * per;
        if (t * 16 + (r & 15) < a.B)
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
            if (n < a.N) st_dev(&a.out_f32[(size_t)b * a.ld_out + n], acc[t][0][i] + (a.bias ? a.bias[n] : 0.f));
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
          store4_frag<T, true>(a.act_out, b, n0, a.out_k_blocks, AP, u);
        }
      }
    }
    return;
  }
  if (EPI == EPI_RESID) {
    // x_out = x_in + sum + bias; per-row (sum, sum of squares) of x_out for the next norm
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
            const float v = a.x_in[(size_t)b * a.N + n] + acc[t][0][i] + (a.bias ? a.bias[n] : 0.f);
            st_dev(&a.x_resid[(size_t)b * a.N + n], v);
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
    if (!arrive_last(&a.counters[ngroups], ngroups, &s_flag)) return;
    {
      // thread (slice = tid / 32, b = tid % 32) sums groups slice, slice + 8, ... in order; the 8
      // slices are then added in order, so the result does not depend on scheduling
      const int b = tid & 31, slice = tid >> 5;
      float t1 = 0.f, t2 = 0.f;
      if (b < a.B) {
#pragma unroll 4
        for (int g = slice; g < ngroups; g += 8) {
          t1 += ld_dev(&a.stat_part[((size_t)g * 32 + b) * 2 + 0]);
          t2 += ld_dev(&a.stat_part[((size_t)g * 32 + b) * 2 + 1]);
        }
      }
      fin_f[slice][b][0] = t1, fin_f[slice][b][1] = t2;
      __syncthreads();
      if (tid < a.B) {
        float u1 = 0.f, u2 = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) u1 += fin_f[q][tid][0], u2 += fin_f[q][tid][1];
        const float inv = 1.0f / (float)a.N;
        float mean = u1 * inv, ms = u2 * inv;
        float rstd;
        if (a.rms) {
          rstd = rsqrtf(ms + a.eps);
          mean = 0.f;
        } else {
          rstd = rsqrtf(fmaxf(ms - mean * mean, 0.f) + a.eps);
        }
        st_dev(&a.stats_out[tid * 2 + 0], mean);
        st_dev(&a.stats_out[tid * 2 + 1], rstd);
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
    if (!arrive_last(&a.counters[ngroups], ngroups, &s_flag)) return;
    {
      // thread (slice = tid / 32, b = tid % 32) scans groups slice, slice + 8, ...; ties go to the
      // lowest index whatever the order, so the merge over slices is order-independent
      const int b = tid & 31, slice = tid >> 5;
      float bv = -INFINITY;
      int bi = INT_MAX;
      if (b < a.B) {
#pragma unroll 4
        for (int g = slice; g < ngroups; g += 8) {
          const float ov = ld_dev(&a.am_val[(size_t)g * 32 + b]);
          const int oi = ld_dev(&a.am_idx[(size_t)g * 32 + b]);
          if (ov > bv || (ov == bv && oi < bi)) bv = ov, bi = oi;
        }
      }
      fin_f[slice][b][0] = bv, fin_i[slice][b] = bi;
      __syncthreads();
      if (tid < a.B) {
        bv = fin_f[0][tid][0], bi = fin_i[0][tid];
#pragma unroll
        for (int q = 1; q < 8; ++q) {
          const float ov = fin_f[q][tid][0];
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

}  // namespace ss
