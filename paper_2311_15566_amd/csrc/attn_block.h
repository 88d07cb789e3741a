// One block's share of decode attention, as a device function.
#pragma once
#include <math.h>

#include "kernels.h"

namespace ss {

// T: cache element type; AT: element type of the operand of the GEMM that consumes the output
template <typename T, int DH> struct RowGeom {
  static constexpr int EPL = Elem<T>::kPerLane;      // elements per lane (16 bytes)
  static constexpr int LPR = DH / EPL;               // lanes per cache row
  static constexpr int G = 64 / LPR;                 // rows per wave-wide load
};

template <typename T>
__device__ __forceinline__ void unpack16(const u32x4 &raw, float *out);
template <>
__device__ __forceinline__ void unpack16<float>(const u32x4 &raw, float *out) {
  f32x4 f = __builtin_bit_cast(f32x4, raw);
  out[0] = f[0], out[1] = f[1], out[2] = f[2], out[3] = f[3];
}
template <>
__device__ __forceinline__ void unpack16<bf16_t>(const u32x4 &raw, float *out) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[2 * i] = __uint_as_float(raw[i] << 16);
    out[2 * i + 1] = __uint_as_float(raw[i] & 0xffff0000u);
  }
}

template <>
__device__ __forceinline__ void unpack16<f16_t>(const u32x4 &raw, float *out) {
  typedef _Float16 h8 __attribute__((ext_vector_type(8)));
  h8 h = __builtin_bit_cast(h8, raw);
#pragma unroll
  for (int i = 0; i < 8; ++i) out[i] = (float)h[i];
}

// ---------------------------------------------------------------------------
// decode attention.  grid = (B*Hs, splits); block = NWV waves.
// Block (bh, s) covers committed rows [s*rpb, min((s+1)*rpb, n)); a lane group of LPR lanes
// owns one row at a time and keeps its own running (max, sum, acc); groups, waves and then
// splits are merged with the usual rescaling.  The last block to arrive for (b, h) also
// scores the new token from registers, writes its key/value as cache row n and emits the
// head output.  Blocks past the live splits exit at once.
// ---------------------------------------------------------------------------
template <int NWV>
struct AttnShared {
  float sq[128];
  float sm_m[NWV], sm_l[NWV];
  float sm_acc[NWV][128];
  float sm_red[4];
  float2 st[NWV];   // raw q|k|v: the waves' shares of the row's (sum, sum of squares)
  int flag;
};

template <typename T, typename AT, int DH, int NWV, bool RAW>
__device__ __forceinline__ void decode_attn_block(const DecodeAttnArgs &a, const int bh, const int sp,
                                                  AttnShared<NWV> &sh) {
  typedef RowGeom<T, DH> Gm;
  constexpr int EPL = Gm::EPL, LPR = Gm::LPR, G = Gm::G, U = NWV >= 8 ? 2 : 4;
  auto &sq = sh.sq;
  auto &sm_m = sh.sm_m;
  auto &sm_l = sh.sm_l;
  auto &sm_acc = sh.sm_acc;
  auto &sm_red = sh.sm_red;
  int &s_flag = sh.flag;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = bh / a.Hs, h = bh - b * a.Hs;
  const int n = a.lens[b];
  if (n >= a.Smax) return;  // a full cache has no row to append to (the host refuses such a step; a replayed capture may not)
  const int live_splits = max(1, (n + a.rows_per_block - 1) / a.rows_per_block);
  if (sp >= live_splits) return;
  const int HD = a.Hs * DH;
  const float scale = rsqrtf((float)DH);
  const float2 *tab = a.rope ? a.rope + (size_t)n * (DH / 2) : nullptr;
  const float *qraw = a.qkv + (size_t)b * 3 * HD + h * DH;
  const int qparts = a.qkv_parts > 1 ? a.qkv_parts : 1;
  const int c = lane % LPR, g = lane / LPR;
  const int r0 = sp * a.rows_per_block;
  const int r1 = min(r0 + a.rows_per_block, n);
  const char *kbase = a.k_cache + b * a.row_stride + h * a.head_stride;
  const char *vbase = a.v_cache + b * a.row_stride + h * a.head_stride;
  constexpr int ROWB = DH * (int)sizeof(T);

  float qf[EPL];
  float new_k = 0.f, new_v = 0.f;
  float m = -1e30f, l = 0.f, acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.f;

  // register batches of U row groups (K and V), two batches in flight
  auto load = [&](u32x4(&kr)[U], u32x4(&vr)[U], const int base) {
    if (base >= r1) return;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int rr = min(base + u * G + g, r1 - 1);  // clamp: masked in consume, stays inside committed rows
      kr[u] = __builtin_nontemporal_load((const u32x4 *)(kbase + (size_t)rr * ROWB) + c);
      vr[u] = __builtin_nontemporal_load((const u32x4 *)(vbase + (size_t)rr * ROWB) + c);
    }
  };
  auto consume = [&](u32x4(&kr)[U], u32x4(&vr)[U], const int base) {
    if (base >= r1) return;
    float s[U];
    float mb = -1e30f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float kf[EPL];
      unpack16<T>(kr[u], kf);
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) d += qf[e] * kf[e];
#pragma unroll
      for (int off = 1; off < LPR; off <<= 1) d += __shfl_xor(d, off);
      s[u] = base + u * G + g < r1 ? d * scale : -INFINITY;
      mb = fmaxf(mb, s[u]);
    }
    const float mn = fmaxf(m, mb);
    const float alpha = __expf(m - mn);
    l *= alpha;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] *= alpha;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float p = __expf(s[u] - mn);
      l += p;
      float vf[EPL];
      unpack16<T>(vr[u], vf);
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[e] += p * vf[e];
    }
    m = mn;
  };
  {
    constexpr int STRIDE = NWV * U * G;
    u32x4 kA[U], vA[U], kB[U], vB[U];
    int base = r0 + wave * (U * G);
    // Raw q|k|v (RAW: a.norm_dim > 0; the GEMM left the normalisation to this kernel; an instance of its own, so that
    // the other one carries none of this): the row's mean and 1/std from the producer's partial sums, thread t adding
    // partials t, t + threads, ...; lanes by a butterfly, waves in order: a fixed order.  These requests (one or two
    // a thread, L2 hits) go out BEFORE the cache rows: loads return in order, and behind the rows they would come back
    // only when the rows have.  (Hoisting the requests for the partial q|k|v sums as well made the kernel slower.)
    // (Inside the RAW instance the flag is read from the arguments all the same: with a compile-time flag the compiler
    // arranged the requests differently and the kernel took 21.4 instead of 20.2 us on the OPT-66B shape.)
    const bool raw = RAW && a.norm_dim > 0;
    float mean = 0.f, rstd = 1.f;
    f32x4 sv = {0.f, 0.f, 0.f, 0.f};
    if (raw)
      for (int gi = tid; gi < a.stat_groups; gi += NWV * 64) sv += ((const f32x4 *)a.stat_in)[(size_t)gi * 32 + b];
    // cache rows do not depend on this step's q: request them first, then stage q
    load(kA, vA, base);
    load(kB, vB, base + STRIDE);
    if (raw && a.stat_groups > 0) {
      float s1 = sv[0] + sv[2], s2 = sv[1] + sv[3];
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) s1 += __shfl_xor(s1, off), s2 += __shfl_xor(s2, off);
      if (lane == 0) sh.st[wave] = make_float2(s1, s2);
      __syncthreads();
      float u1 = 0.f, u2 = 0.f;
#pragma unroll
      for (int w2 = 0; w2 < NWV; ++w2) u1 += sh.st[w2].x, u2 += sh.st[w2].y;
      const float inv = 1.0f / (float)a.norm_dim;
      const float ms = u2 * inv;
      if (a.rms) {
        rstd = rsqrtf(ms + a.eps);
      } else {
        mean = u1 * inv;
        rstd = rsqrtf(fmaxf(ms - mean * mean, 0.f) + a.eps);
        // the next producer centres on this norm's mean (one thread per batch row)
        if (a.publish && a.cen && h == 0 && sp == 0 && tid == 0) a.cen[b] = a.cen[b] + mean;
      }
    }
    float kn = 0.f, vraw = 0.f;  // the new token's (rotated) key and value element of thread e
    if (tid < DH) {
      // q | k | v of the new token: the GEMM's partial sums (it may have cut K into slices), all requested at
      // once and then added in slice order; q and k rotated to position n (half-split pairing) when the
      // model has a rotation table
      constexpr int HALF = DH / 2;
      const int e = tid, eo = e < HALF ? e + HALF : e - HALF;
      float pq[kQkvParts], pk[kQkvParts], pv[kQkvParts], pqo[kQkvParts], pko[kQkvParts];
#pragma unroll
      for (int p = 0; p < kQkvParts; ++p) {
        if (p < qparts) {  // block-uniform
          const float *src = qraw + (size_t)p * a.qkv_stride;
          pq[p] = src[e], pk[p] = src[HD + e], pv[p] = src[2 * HD + e];
          pqo[p] = src[eo], pko[p] = src[HD + eo];  // the rotation partners (unused without a table)
        }
      }
      // (raw q|k|v: the folded vectors of the five columns, requested with the partial sums)
      float wgv[5] = {0.f, 0.f, 0.f, 0.f, 0.f}, cbv[5] = {0.f, 0.f, 0.f, 0.f, 0.f};
      if (raw) {
        const int cq = h * DH + e, cqo = h * DH + eo;
        const int col[5] = {cq, HD + cq, 2 * HD + cq, cqo, HD + cqo};
#pragma unroll
        for (int i = 0; i < 5; ++i) {
          if (a.wg) wgv[i] = a.wg[col[i]];
          if (a.cb) cbv[i] = a.cb[col[i]];
        }
      }
      float qe = pq[0], ke = pk[0], qo = pqo[0], ko = pko[0];
      vraw = pv[0];
#pragma unroll
      for (int p = 1; p < kQkvParts; ++p)
        if (p < qparts) qe += pq[p], ke += pk[p], vraw += pv[p], qo += pqo[p], ko += pko[p];
      if (raw) {
        qe = rstd * (qe - mean * wgv[0]) + cbv[0], ke = rstd * (ke - mean * wgv[1]) + cbv[1];
        vraw = rstd * (vraw - mean * wgv[2]) + cbv[2];
        qo = rstd * (qo - mean * wgv[3]) + cbv[3], ko = rstd * (ko - mean * wgv[4]) + cbv[4];
      }
      if (tab) {
        const float2 cs = tab[e < HALF ? e : e - HALF];
        if (e < HALF) qe = qe * cs.x - qo * cs.y, ke = ke * cs.x - ko * cs.y;
        else qe = qo * cs.y + qe * cs.x, ke = ko * cs.y + ke * cs.x;
      }
      kn = ke;
      sq[tid] = qe;
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < EPL; ++e) qf[e] = sq[c * EPL + e];
    for (; base < r1; base += 2 * STRIDE) {
      consume(kA, vA, base);
      load(kA, vA, base + 2 * STRIDE);
      consume(kB, vB, base + STRIDE);
      load(kB, vB, base + 3 * STRIDE);
    }
    new_k = kn, new_v = vraw;
  }
  // merge the G lane groups of the wave
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
    const float mo = __shfl_xor(m, off), lo = __shfl_xor(l, off);
    const float mn = fmaxf(m, mo);
    const float f0 = __expf(m - mn), f1 = __expf(mo - mn);
    l = l * f0 + lo * f1;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = acc[e] * f0 + __shfl_xor(acc[e], off) * f1;
    m = mn;
  }
  if (lane < LPR) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) sm_acc[wave][lane * EPL + e] = acc[e];
    if (lane == 0) sm_m[wave] = m, sm_l[wave] = l;
  }
  __syncthreads();
  // merge the waves; thread e owns output dim e
  float M = -1e30f, Lsum = 0.f, A = 0.f;
  if (tid < DH) {
#pragma unroll
    for (int w = 0; w < NWV; ++w) M = fmaxf(M, sm_m[w]);
#pragma unroll
    for (int w = 0; w < NWV; ++w) {
      const float f = __expf(sm_m[w] - M);
      Lsum += sm_l[w] * f;
      A += sm_acc[w][tid] * f;
    }
  }
  float *part = a.part + ((size_t)bh * a.splits) * (DH + 4);
  if (live_splits > 1) {
    if (tid < DH) {
      float *p = part + (size_t)sp * (DH + 4);
      st_dev(p + tid, A);
      if (tid == 0) st_dev(p + DH, M), st_dev(p + DH + 1, Lsum);
    }
    if (!arrive_last(&a.counters[bh], live_splits, &s_flag)) return;
    if (tid < DH) {
      // the partials in batches of eight splits, every load of a batch requested before the first is used
      // (one round trip a batch); same order of additions as split by split, with a running maximum
      M = -1e30f, Lsum = 0.f, A = 0.f;
      for (int s0 = 0; s0 < live_splits; s0 += 8) {
        float pm[8], pl[8], pa[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          if (s0 + i < live_splits) {  // block-uniform
            const float *p = part + (size_t)(s0 + i) * (DH + 4);
            pm[i] = ld_dev(p + DH), pl[i] = ld_dev(p + DH + 1), pa[i] = ld_dev(p + tid);
          }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          if (s0 + i < live_splits) {
            const float mn = fmaxf(M, pm[i]);
            const float f0 = __expf(M - mn), f1 = __expf(pm[i] - mn);
            Lsum = Lsum * f0 + pl[i] * f1;
            A = A * f0 + pa[i] * f1;
            M = mn;
          }
        }
      }
    }
  }
  // the new token: append as row n (not committed until the step's last kernel), attend to itself
  float vnew = 0.f, prod = 0.f;
  if (tid < DH) {
    const T kt = Elem<T>::from_f32(new_k);
    const T vt = Elem<T>::from_f32(new_v);
    ((T *)(a.k_cache + b * a.row_stride + h * a.head_stride + (size_t)n * ROWB))[tid] = kt;
    ((T *)(a.v_cache + b * a.row_stride + h * a.head_stride + (size_t)n * ROWB))[tid] = vt;
    vnew = Elem<T>::to_f32(vt);
    prod = sq[tid] * Elem<T>::to_f32(kt);
  }
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) prod += __shfl_xor(prod, off);
  if (lane == 0 && wave < 4) sm_red[wave] = prod;
  __syncthreads();
  if (tid < DH) {
    float sn = 0.f;
#pragma unroll
    for (int w = 0; w < (DH + 63) / 64; ++w) sn += sm_red[w];
    sn *= scale;
    const float mn = fmaxf(M, sn);
    const float f0 = __expf(M - mn), p = __expf(sn - mn);
    const float Lf = Lsum * f0 + p;
    const float o = (A * f0 + p * vnew) / Lf;
    // neighbouring dims pair up so that the operand buffer is written in whole words
    const float o_next = __shfl_xor(o, 1);
    if (sizeof(AT) == 4) {
      float *p = (float *)a.o_out + frag_offset<AT>(b, h * DH + tid, HD / Elem<AT>::kFragK);
      st_dev(p, o);
    } else if ((tid & 1) == 0) {
      const AT w[2] = {Elem<AT>::from_f32(o), Elem<AT>::from_f32(o_next)};
      uint32_t word;
      __builtin_memcpy(&word, w, 4);
      st_dev((uint32_t *)((AT *)a.o_out + frag_offset<AT>(b, h * DH + tid, HD / Elem<AT>::kFragK)), word);
    }
  }
}

}  // namespace ss
