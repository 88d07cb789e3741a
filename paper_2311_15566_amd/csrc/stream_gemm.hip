// The weight-streaming GEMM of the decode step and the fold of a norm's gamma / beta into
// per-output vectors (see StreamGemmArgs).
#include <limits.h>
#include <math.h>
#include <stdlib.h>

#include "kernels.h"
#include "mma.h"

namespace ss {

namespace {

constexpr int U = 2;      // fragments per register batch; two batches in flight

template <int NB, int KSM, int NW>
struct GemmShared {
  f32x4 red[KSM][NW][NB][64];    // per K slice: the wave's sums [weight tile][batch tile][lane]
  float stat[KSM * NB * 16 * 2]; // row sums per wave: [wave][batch tile][row][2]
  float lg_v[NW][NB * 16];       // logits: best value / index per weight tile and row
  int lg_i[NW][NB * 16];
};

}  // namespace

// grid = groups x K slices, block = a.ks waves.  Group g owns the weight tiles of units
// [g * units / n_blocks, (g + 1) * units / n_blocks) (a unit is one 16-row tile, or a gate/up pair of
// them): at most NW tiles, fewer where the units do not divide evenly, so every group's share of the
// matrix differs by one unit at most.  Wave s streams k blocks [s * per, (s + 1) * per) of the block's
// K slice for all its tiles in register batches of U fragments per tile, two batches in flight, and
// shares the activation fragments between the tiles.
// KSM: waves per block at most.  NW: weight tiles per block at most.
template <typename T, int NB, bool GLU, int EPI, int KSM, int NW>
__global__ void __launch_bounds__(KSM * 64, 2) stream_gemm(StreamGemmArgs a) {
  typedef typename Operand<T>::type OT;  // element type of the activation operands
  constexpr int RB = NB * 16;
  constexpr int TU = GLU ? 2 : 1;          // weight tiles per unit: the tiles one epilogue item combines
  constexpr int NU = NW / TU;              // units per block at most
  constexpr int NITEMS = NU * NB;          // epilogue items: (unit, batch tile)
  constexpr int NIT = (NITEMS + 3) / 4;    // items per wave at most (a block has 4 or 8 waves)
  static_assert(NW % TU == 0, "a block holds whole units");
  __shared__ GemmShared<NB, KSM, NW> sh;
  const int tid = threadIdx.x, lane = tid & 63, ks = tid >> 6, KS = blockDim.x >> 6;
  // Block -> (group, K slice).  EPI_F32 with a.k_split = S > 1: S blocks per group, each over one
  // slice of K; they leave S partial outputs (out_f32 + kh * part_stride) that the consumer adds up
  // in slice order, so no block waits for another.  Slices after the first contribute acc * rstd
  // only (no mean, no bias).
  const int S = (EPI == EPI_F32 && a.k_split > 1) ? a.k_split : 1;
  const int grp = blockIdx.x / S, kh = blockIdx.x - grp * S;
  const int units = a.row_tiles / TU;
  const int u0 = (int)((long)grp * units / a.n_blocks), u1 = (int)((long)(grp + 1) * units / a.n_blocks);
  const int tile0 = u0 * TU;
  const int cnt = (u1 - u0) * TU;          // tiles of this block (<= NW: checked on the host)
  const int k_slice = (a.k_blocks + S - 1) / S;
  const int k_lo = kh * k_slice, k_hi = min(a.k_blocks, k_lo + k_slice);
  const int per = (k_hi - k_lo + KS - 1) / KS;
  const int k0 = k_lo + ks * per, k1 = min(k_hi, k0 + per);
  const int r = lane & 15, q4 = (lane >> 4) * 4;

  bool tile_ok[NW];
  const u32x4 *wp[NW];
#pragma unroll
  for (int j = 0; j < NW; ++j) {
    tile_ok[j] = j < cnt;
    wp[j] = (const u32x4 *)a.w + (size_t)(tile0 + j) * a.k_blocks * 64 + lane;
  }
  bool row_ok[NB];
  const u32x4 *ap[NB];
#pragma unroll
  for (int t = 0; t < NB; ++t) {
    row_ok[t] = t * 16 + r < a.B;
    ap[t] = (const u32x4 *)a.act + (size_t)t * a.k_blocks * 64 + lane;
  }

  // what the epilogue needs from memory is requested first, so that it has long arrived.
  // Epilogue item i = (unit i % NU, batch tile i / NU); wave ks takes items ks, ks + KS, ...
  bool it_live[NIT];          // the item exists and this lane's row and outputs are inside the problem
  int it_b[NIT], it_n0[NIT];  // this lane's batch row and the first of its four outputs
  f32x4 e_wg[NIT][TU], e_cb[NIT][TU], e_x[NIT], e_g[NIT];
  float e_cen = 0.f;  // EPI_RESID: the centre of the operand it writes; a publishing consumer: the centre of the one it reads
  {
    const int b0 = (ks / NU) * 16 + r;  // the row of this wave's first item
    if (ks < NITEMS && a.cen && b0 < a.B && (EPI == EPI_RESID || (a.publish && grp == 0 && kh == 0))) e_cen = a.cen[b0];
  }
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int item = ks + it * KS;
    const int je = item % NU, te = item / NU;
    const int b = te * 16 + r;
    const int wrow = (tile0 + je * TU) * 16 + q4;            // first of its four weight rows (gate rows for a pair)
    const int n0 = GLU ? (u0 + je) * 16 + q4 : wrow;
    it_b[it] = b, it_n0[it] = n0;
    it_live[it] = item < NITEMS && je * TU < cnt && b < a.B && n0 < a.N;
    e_x[it] = f32x4{0.f, 0.f, 0.f, 0.f}, e_g[it] = f32x4{1.f, 1.f, 1.f, 1.f};
#pragma unroll
    for (int jj = 0; jj < TU; ++jj) {
      e_wg[it][jj] = e_cb[it][jj] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (it_live[it] && kh == 0) {
        if (a.wg) e_wg[it][jj] = *(const f32x4 *)(a.wg + wrow + jj * 16);
        if (a.cb) e_cb[it][jj] = *(const f32x4 *)(a.cb + wrow + jj * 16);
      }
    }
    if (EPI == EPI_RESID && it_live[it]) {
      e_x[it] = *(const f32x4 *)(a.x_in + (size_t)b * a.N + n0);
      if (a.act_out) e_g[it] = *(const f32x4 *)(a.g_out + n0);
    }
    if (EPI == EPI_RESID && it > 0 && item < NITEMS && a.cen && b < a.B && it_b[0] != b) e_cen = e_cen;  // (rows of later items: see below)
  }

  f32x4 acc[NB][NW];
#pragma unroll
  for (int t = 0; t < NB; ++t)
#pragma unroll
    for (int j = 0; j < NW; ++j) acc[t][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  auto load = [&](u32x4(&w)[NW][U], u32x4(&av)[NB][U], int kb) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool ok = kb + u < k1;
#pragma unroll
      for (int j = 0; j < NW; ++j)
        w[j][u] = (ok && tile_ok[j]) ? __builtin_nontemporal_load(wp[j] + (size_t)(kb + u) * 64) : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
      for (int t = 0; t < NB; ++t) av[t][u] = (ok && row_ok[t]) ? ap[t][(size_t)(kb + u) * 64] : u32x4{0u, 0u, 0u, 0u};
    }
  };
  auto use = [&](u32x4(&w)[NW][U], u32x4(&av)[NB][U]) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int j = 0; j < NW; ++j) {
#pragma unroll
        for (int t = 0; t < NB; ++t) acc[t][j] = mma_op<T>(w[j][u], av[t][u], acc[t][j]);
      }
  };

  u32x4 wA[NW][U], aA[NB][U], wB[NW][U], aB[NB][U];
  load(wA, aA, k0);
  load(wB, aB, k0 + U);

  // Row sums of the normalised input.  The producer left one (sum, sum of squares) pair per 16-row
  // weight tile and row, two tiles to a float4.  Thread (slice, row) adds float4s slice,
  // slice + nsl, ...; the slices of a wave are then added by a butterfly over its lanes and the
  // waves in order in the epilogue.  The first SR float4s are requested here, behind the first
  // weight batches, and added after the main loop, when they have long arrived: nothing waits
  // for them now.
  constexpr bool NORMED = EPI != EPI_RESID;
  constexpr int SR = NORMED ? (GLU ? 2 : 4) : 0;
  // (the split of the partials over threads depends on the batch size only, so the sums come out
  // the same whatever the launch shape: 8 or 16 rows a slice, a thread takes that row of every
  // batch tile of the block)
  const int rbl = a.B <= 8 ? 8 : 16;
  const int nsl = blockDim.x / rbl;
  const int st_slice = tid / rbl, st_loc = tid % rbl;
  const f32x4 *st_p = (const f32x4 *)a.stat_in + st_loc;
  f32x4 st_v[NB][SR > 0 ? SR : 1];
  if (NORMED) {
#pragma unroll
    for (int t = 0; t < NB; ++t)
#pragma unroll
      for (int i = 0; i < SR; ++i) {
        const int g = st_slice + i * nsl;
        st_v[t][i] = (t * 16 + st_loc < a.B && g < a.stat_groups) ? st_p[(size_t)g * 32 + t * 16]
                                                                 : f32x4{0.f, 0.f, 0.f, 0.f};
      }
  }

  for (int kb = k0; kb < k1; kb += 2 * U) {
    use(wA, aA);
    load(wA, aA, kb + 2 * U);
    use(wB, aB);
    load(wB, aB, kb + 3 * U);
  }

  if (NORMED && a.stat_groups > 0) {
#pragma unroll
    for (int t = 0; t < NB; ++t) {
      f32x4 sv = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < SR; ++i) sv += st_v[t][i];
      if (t * 16 + st_loc < a.B)
        for (int g = st_slice + SR * nsl; g < a.stat_groups; g += nsl) sv += st_p[(size_t)g * 32 + t * 16];  // the rest, if any
      // lanes loc, loc + rbl, loc + 2 rbl, ... of the wave hold the slices of row loc
      float s1 = sv[0] + sv[2], s2 = sv[1] + sv[3];
      for (int off = rbl; off < 64; off <<= 1) s1 += __shfl_xor(s1, off), s2 += __shfl_xor(s2, off);
      if (lane < rbl) {
        float *dst = &sh.stat[((ks * NB + t) * 16 + lane) * 2];
        dst[0] = s1, dst[1] = s2;
      }
    }
  }
#pragma unroll
  for (int t = 0; t < NB; ++t)
#pragma unroll
    for (int j = 0; j < NW; ++j) sh.red[ks][j][t][lane] = acc[t][j];
  __syncthreads();

#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int item = ks + it * KS;
    if (item >= NITEMS) break;  // wave-uniform
    const int je = item % NU, te = item / NU;
    const int b = it_b[it], n0 = it_n0[it], bl = te * 16 + r;
    const bool epi_live = it_live[it];
    const bool unit_ok = je * TU < cnt;
    float bv = -INFINITY;  // EPI_LOGITS: this lane's best
    int bi = INT_MAX;
    f32x4 sum[TU];
#pragma unroll
    for (int jj = 0; jj < TU; ++jj) {
      const int j = je * TU + jj;
      f32x4 part[KSM];  // all slices requested before the first is added: one LDS round trip, not KS
#pragma unroll
      for (int s = 0; s < KSM; ++s) part[s] = sh.red[s < KS ? s : 0][j][te][lane];
      sum[jj] = part[0];
#pragma unroll
      for (int s = 1; s < KSM; ++s)
        if (s < KS) sum[jj] += part[s];
    }
    float mean = 0.f, rstd = 1.f;  // mean: of the centred rows, i.e. mean(x) - c
    if (NORMED && a.stat_groups > 0) {
      float u1 = 0.f, u2 = 0.f;
      const int br = r < rbl ? r : 0;  // rows past the batch are masked later
      float2 sp[KSM];
#pragma unroll
      for (int s = 0; s < KSM; ++s) sp[s] = *(const float2 *)&sh.stat[(((s < KS ? s : 0) * NB + te) * 16 + br) * 2];
#pragma unroll
      for (int s = 0; s < KSM; ++s)
        if (s < KS) u1 += sp[s].x, u2 += sp[s].y;
      const float inv = 1.0f / (float)a.norm_dim;
      const float ms = u2 * inv;
      if (a.rms) {
        rstd = rsqrtf(ms + a.eps);
      } else {
        mean = u1 * inv;
        rstd = rsqrtf(fmaxf(ms - mean * mean, 0.f) + a.eps);
        // the next producer centres on this norm's mean (one lane per row, first block, first unit)
        if (a.publish && a.cen && grp == 0 && kh == 0 && je == 0 && lane < 16 && b < a.B) a.cen[b] = (it == 0 ? e_cen : a.cen[b]) + mean;
      }
    }
    float h[TU][4];  // the product with normalisation and bias applied
#pragma unroll
    for (int jj = 0; jj < TU; ++jj)
#pragma unroll
      for (int i = 0; i < 4; ++i) h[jj][i] = rstd * (sum[jj][i] - mean * e_wg[it][jj][i]) + e_cb[it][jj][i];

    if (EPI == EPI_F32) {
      if (epi_live) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (n0 + i < a.N) a.out_f32[(size_t)kh * a.part_stride + (size_t)b * a.ld_out + n0 + i] = h[0][i];
      }
    } else if (EPI == EPI_ACT || EPI == EPI_SWIGLU) {
      if (epi_live) {
        float u[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) u[i] = GLU ? silu_f(h[0][i]) * h[TU - 1][i] : act_apply(a.act_kind, h[0][i]);
        store4_frag<OT, false>(a.act_out, b, n0, a.out_k_blocks, u);
      }
    } else if (EPI == EPI_RESID) {
      float s1 = 0.f, s2 = 0.f;
      if (epi_live) {
        const float cen = it == 0 ? e_cen : (a.cen ? a.cen[b] : 0.f);
        float v[4], g[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          v[i] = e_x[it][i] + h[0][i];
          const float t = v[i] - cen;
          s1 += t, s2 += t * t;
          g[i] = t * e_g[it][i];
        }
        *(f32x4 *)(a.x_out + (size_t)b * a.N + n0) = f32x4{v[0], v[1], v[2], v[3]};
        if (a.act_out) store4_frag<OT, false>(a.act_out, b, n0, a.out_k_blocks, g);
      }
      if (a.act_out) {  // partial row sums of this weight tile's 16 features
        s1 += __shfl_xor(s1, 16), s2 += __shfl_xor(s2, 16);
        s1 += __shfl_xor(s1, 32), s2 += __shfl_xor(s2, 32);
        if (lane < 16 && unit_ok && b < a.B)  // weight tile tile0 + je: half (tile & 1) of float4 number tile >> 1
          ((float2 *)a.stat_out)[((size_t)((tile0 + je) >> 1) * 32 + b) * 2 + ((tile0 + je) & 1)] = make_float2(s1, s2);
      }
    } else {  // EPI_LOGITS
      if (epi_live) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (n0 + i < a.N) {
            if (a.out_f32) a.out_f32[(size_t)b * a.ld_out + n0 + i] = h[0][i];
            if (h[0][i] > bv) bv = h[0][i], bi = n0 + i;
          }
        }
      }
#pragma unroll
      for (int off = 16; off <= 32; off <<= 1) {
        const float ov = __shfl_xor(bv, off);
        const int oi = __shfl_xor(bi, off);
        if (ov > bv || (ov == bv && oi < bi)) bv = ov, bi = oi;
      }
      if (lane < 16) sh.lg_v[je][bl] = bv, sh.lg_i[je][bl] = bi;
    }
  }
  if (EPI != EPI_LOGITS) return;

  // ---- greedy choice over the vocabulary: this block's best per batch row; the step's last kernel
  // (choose_and_commit) picks among the blocks.  No block waits for another and nothing is counted:
  // a device-wide counter that every block bumps and reads back made the kernel 14 us longer.
  __syncthreads();
  if (tid < RB && tid < a.B) {
    float bv = sh.lg_v[0][tid];
    int bi = sh.lg_i[0][tid];
#pragma unroll
    for (int j = 1; j < NU; ++j) {
      if (j >= cnt) break;
      const float ov = sh.lg_v[j][tid];
      const int oi = sh.lg_i[j][tid];
      if (ov > bv || (ov == bv && oi < bi)) bv = ov, bi = oi;
    }
    a.am_val[(size_t)tid * a.n_blocks + grp] = bv;   // [row][block]: a row's candidates are contiguous
    a.am_idx[(size_t)tid * a.n_blocks + grp] = bi;
  }
}

// ---------------------------------------------------------------------------
// wg[row] = sum_k W[row, k] gamma[k],  cb[row] = sum_k W[row, k] beta[k] + bias[row]
// one wave per weight tile, sums in double
// ---------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) fold_norm(const u32x4 *__restrict__ w, int row_tiles, int k_blocks,
                                                 const float *__restrict__ gamma, const float *__restrict__ beta,
                                                 const float *__restrict__ bias, float *__restrict__ wg,
                                                 float *__restrict__ cb) {
  typedef typename Operand<T>::type WT;  // the fragments hold the weights in the operand type
  constexpr int PL = Elem<T>::kPerLane, FK = Elem<T>::kFragK;
  const int lane = threadIdx.x & 63, tile = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (tile >= row_tiles) return;
  const int r = lane & 15, kq = lane >> 4;
  double sg = 0.0, sb = 0.0;
  for (int kb = 0; kb < k_blocks; ++kb) {
    const u32x4 raw = w[((size_t)tile * k_blocks + kb) * 64 + lane];
    WT e[PL];
    __builtin_memcpy(e, &raw, 16);
#pragma unroll
    for (int i = 0; i < PL; ++i) {
      const int k = kb * FK + kq * PL + i;
      const double wv = (double)Elem<WT>::to_f32(e[i]);
      if (gamma) sg += wv * (double)gamma[k];
      if (beta) sb += wv * (double)beta[k];
    }
  }
  sg += __shfl_xor(sg, 16), sb += __shfl_xor(sb, 16);
  sg += __shfl_xor(sg, 32), sb += __shfl_xor(sb, 32);
  if (lane < 16) {
    const int row = tile * 16 + r;
    if (gamma && wg) wg[row] = (float)sg;
    if (cb) cb[row] = (float)(sb + (bias ? (double)bias[row] : 0.0));
  }
}

ss_status launch_fold_norm(int dtype, const void *w, int row_tiles, int k_blocks, const float *gamma, const float *beta,
                           const float *bias, float *wg, float *cb, hipStream_t st) {
  if (!w || row_tiles < 1 || k_blocks < 1) SS_FAIL(SS_EINVAL, "fold: bad arguments");
  const dim3 grid(ceil_div(row_tiles, 4)), block(256);
  if (dtype == SS_DTYPE_BF16)
    hipLaunchKernelGGL(fold_norm<bf16_t>, grid, block, 0, st, (const u32x4 *)w, row_tiles, k_blocks, gamma, beta, bias, wg, cb);
  else
    hipLaunchKernelGGL(fold_norm<float>, grid, block, 0, st, (const u32x4 *)w, row_tiles, k_blocks, gamma, beta, bias, wg, cb);
  SS_HIP(hipGetLastError());
  return SS_OK;
}

}  // namespace ss
