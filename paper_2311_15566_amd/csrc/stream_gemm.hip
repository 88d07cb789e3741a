// The weight-streaming GEMM of the decode step and the fold of a norm's gamma / beta into
// per-output vectors (see StreamGemmArgs).
#include <limits.h>
#include <math.h>
#include <stdlib.h>

#include <atomic>

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

// grid = groups x K slices, block = a.ks waves.  The units (a unit is one 16-row weight tile, or a
// gate/up pair of them) are shared out over the n_blocks groups in order, units / n_blocks each and
// one more for the first units % n_blocks groups: at most NW tiles a group, and no two groups' shares
// differ by more than one unit.  Wave s streams k blocks [s * per, (s + 1) * per) of the block's
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
  // The waves' sums meet in LDS.  The widest instance (6 tiles x 2 batch tiles) needs more than the 64 KiB a
  // kernel may declare, and takes its LDS at launch instead.
  typedef GemmShared<NB, KSM, NW> Shared;
  constexpr bool DYN_LDS = sizeof(Shared) > 64 * 1024;
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  __shared__ __align__(16) unsigned char fix_lds[DYN_LDS ? 16 : sizeof(Shared)];
  Shared &sh = *reinterpret_cast<Shared *>(DYN_LDS ? dyn_lds : fix_lds);
  const int tid = threadIdx.x, lane = tid & 63, KS = blockDim.x >> 6;
  // The wave's number as a scalar: everything derived from it (its k range, its epilogue items) is then
  // wave-uniform for the compiler too, and the branches on it are real branches.  (A matrix-core
  // instruction runs whatever the lane mask says, so it must never sit in a block that is merely
  // masked off: with a k range the compiler takes for lane-dependent, a skipped batch's products
  // were added all the same, from registers nothing had been loaded into.)
  const int ks = __builtin_amdgcn_readfirstlane(tid >> 6);
  // Block -> (group, K slice).  EPI_F32 with a.k_split = S > 1: S blocks per group, each over one
  // slice of K; they leave S partial outputs (out_f32 + kh * part_stride) that the consumer adds up
  // in slice order, so no block waits for another.  Slices after the first contribute acc * rstd
  // only (no mean, no bias).
  int grp = blockIdx.x, kh = 0;
  if (EPI == EPI_F32 && a.k_split > 1) grp = blockIdx.x / a.k_split, kh = blockIdx.x - grp * a.k_split;
  // the first u_rem groups own u_base + 1 units, the others u_base (no division here: every block would pay for it)
  const int u0 = grp * a.u_base + min(grp, a.u_rem);
  const int tile0 = u0 * TU;
  const int cnt = (a.u_base + (grp < a.u_rem ? 1 : 0)) * TU;  // tiles of this block (<= NW: checked on the host)
  const int k_lo = kh * a.k_slice, k_hi = min(a.k_blocks, k_lo + a.k_slice);
  const int per = (k_hi - k_lo + KS - 1) >> (KS == 8 ? 3 : 2);  // KS is 4 or 8
  const int k0 = k_lo + ks * per, k1 = min(k_hi, k0 + per);
  const int r = lane & 15, q4 = (lane >> 4) * 4;

  // Every load of the main loop is unconditional: a tile past the block's share streams the block's
  // first tile again (its sums are never stored), a batch row past the batch and a k block past the
  // wave's range read a fragment of zeros.  Loads under lane- or tile-dependent branches make the
  // compiler wait for them where the branches meet, in the middle of the requests.
  const u32x4 *wp[NW];
#pragma unroll
  for (int j = 0; j < NW; ++j) wp[j] = (const u32x4 *)a.w + (size_t)(tile0 + (j < cnt ? j : 0)) * a.k_blocks * 64 + lane;
  bool row_ok[NB];
  const u32x4 *ap[NB];
#pragma unroll
  for (int t = 0; t < NB; ++t) {
    row_ok[t] = t * 16 + r < a.B;
    ap[t] = (const u32x4 *)a.act + (size_t)t * a.k_blocks * 64 + lane;
  }
  const u32x4 *zfrag = (const u32x4 *)a.zero_frag + lane;  // 1 KiB of zeros (in the shard's memory: a pointer of the same kind as the others)

  // What the epilogue needs from memory is requested first, so that it has long arrived.  Every
  // request is unconditional (where there is nothing to read it goes to the start of the weights,
  // always valid, and the value is dropped in the epilogue): a load under a branch makes the
  // compiler wait for it where the branches meet, i.e. before the weight stream starts.
  // Epilogue item i = (unit i % NU, batch tile i / NU); wave ks takes items ks, ks + KS, ...
  bool it_live[NIT];          // the item exists and this lane's row and outputs are inside the problem
  int it_b[NIT], it_n0[NIT];  // this lane's batch row and the first of its four outputs
  f32x4 e_wg[NIT][TU], e_cb[NIT][TU], e_x[NIT], e_g[NIT];
  float e_cen[NIT];           // EPI_RESID: the centre of the operand it writes; a publishing consumer: the centre of the one it reads
  const float *dummy = (const float *)a.w;
  const bool first_slice = kh == 0;
  const bool want_cen = a.cen && (EPI == EPI_RESID || (a.publish && grp == 0 && first_slice));
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int item = ks + it * KS;
    const int je = item % NU, te = item / NU;
    const int b = te * 16 + r;
    const int wrow = (tile0 + je * TU) * 16 + q4;            // first of its four weight rows (gate rows for a pair)
    const int n0 = GLU ? (u0 + je) * 16 + q4 : wrow;
    it_b[it] = b, it_n0[it] = n0;
    const bool live = item < NITEMS && je * TU < cnt && b < a.B && n0 < a.N;
    it_live[it] = live;
    e_cen[it] = *((want_cen && item < NITEMS && b < a.B) ? a.cen + b : dummy);
#pragma unroll
    for (int jj = 0; jj < TU; ++jj) {
      e_wg[it][jj] = *(const f32x4 *)((live && first_slice && a.wg) ? a.wg + wrow + jj * 16 : dummy);
      e_cb[it][jj] = *(const f32x4 *)((live && first_slice && a.cb) ? a.cb + wrow + jj * 16 : dummy);
    }
    if (EPI == EPI_RESID) {
      e_x[it] = *(const f32x4 *)(live ? a.x_in + (size_t)b * a.N + n0 : dummy);
      e_g[it] = *(const f32x4 *)((live && a.act_out) ? a.g_out + n0 : dummy);
    }
  }

  f32x4 acc[NB][NW];
#pragma unroll
  for (int t = 0; t < NB; ++t)
#pragma unroll
    for (int j = 0; j < NW; ++j) acc[t][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int k_last = max(k1 - 1, k_lo);  // a k block that exists, for requests past the wave's range (the matching activations are zeros)
  auto load = [&](u32x4(&w)[NW][U], u32x4(&av)[NB][U], int kb) {
    if (kb >= k1) return;  // wave-uniform: nothing of this batch is inside the range, and use() skips it too
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool ok = kb + u < k1;
      const size_t off = (size_t)min(kb + u, k_last) * 64;
#pragma unroll
      for (int j = 0; j < NW; ++j) w[j][u] = __builtin_nontemporal_load(wp[j] + off);
#pragma unroll
      for (int t = 0; t < NB; ++t) av[t][u] = *((ok && row_ok[t]) ? ap[t] + off : zfrag);
    }
  };
  auto use = [&](u32x4(&w)[NW][U], u32x4(&av)[NB][U], int kb) {
    if (kb >= k1) return;
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
  constexpr int SR = NORMED ? (NB * NW >= 12 ? 1 : (GLU ? 2 : 4)) : 0;  // (the widest instance has no registers to spare)
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
        st_v[t][i] = *((t * 16 + st_loc < a.B && g < a.stat_groups) ? st_p + (size_t)g * 32 + t * 16 : (const f32x4 *)a.zero_frag);
      }
  }

  for (int kb = k0; kb < k1; kb += 2 * U) {
    use(wA, aA, kb);
    load(wA, aA, kb + 2 * U);
    use(wB, aB, kb + U);
    load(wB, aB, kb + 3 * U);
  }

  if (NORMED && a.stat_groups > 0) {
#pragma unroll
    for (int t = 0; t < NB; ++t) {
      f32x4 sv = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < SR; ++i) sv += st_v[t][i];
      // the rest, if any: four requests at a time (a request per trip would wait for each in turn), added in the same order
      if (t * 16 + st_loc < a.B) {
        for (int g = st_slice + SR * nsl; g < a.stat_groups; g += 4 * nsl) {
          f32x4 more[4];
#pragma unroll
          for (int i = 0; i < 4; ++i)
            more[i] = *(g + i * nsl < a.stat_groups ? st_p + (size_t)(g + i * nsl) * 32 + t * 16 : (const f32x4 *)a.zero_frag);
#pragma unroll
          for (int i = 0; i < 4; ++i) sv += more[i];
        }
      }
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
        if (a.publish && a.cen && grp == 0 && first_slice && je == 0 && lane < 16 && b < a.B) a.cen[b] = e_cen[it] + mean;
      }
    }
    float h[TU][4];  // the product with normalisation and bias applied
    const bool has_wg = epi_live && first_slice && a.wg, has_cb = epi_live && first_slice && a.cb;
#pragma unroll
    for (int jj = 0; jj < TU; ++jj)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        h[jj][i] = rstd * (sum[jj][i] - (has_wg ? mean * e_wg[it][jj][i] : 0.f)) + (has_cb ? e_cb[it][jj][i] : 0.f);

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
        const float cen = a.cen ? e_cen[it] : 0.f;
        float v[4], g[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          v[i] = e_x[it][i] + h[0][i];
          const float t = v[i] - cen;
          s1 += t, s2 += t * t;
          g[i] = a.act_out ? t * e_g[it][i] : 0.f;
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

// units a block owns at most when n_blocks groups share the matrix evenly
int stream_gemm_units_per_block(int epi, const StreamGemmArgs &a) {
  const int units = epi == EPI_SWIGLU ? a.row_tiles / 2 : a.row_tiles;
  return a.n_blocks > 0 ? ceil_div(units, a.n_blocks) : 0;
}

ss_status check_stream_gemm(int dtype, int epi, const StreamGemmArgs &a) {
  if (dtype != SS_DTYPE_BF16 && dtype != SS_DTYPE_F32) SS_FAIL(SS_EINVAL, "decode GEMM: dtype %d", dtype);
  if (a.B < 1 || a.B > 32) SS_FAIL(SS_EINVAL, "decode GEMM: batch %d", a.B);
  const int tu = epi == EPI_SWIGLU ? 2 : 1, units = a.row_tiles / tu;
  if (a.row_tiles < 1 || a.k_blocks < 1 || (a.ks != 4 && a.ks != 8) || a.N < 1 || a.N > a.row_tiles * 16)
    SS_FAIL(SS_EINVAL, "decode GEMM: bad shape (tiles %d, k blocks %d, waves %d, N %d)", a.row_tiles, a.k_blocks, a.ks, a.N);
  // instances: 1, 2 or 3 tiles a block; a gate/up pair; or the wide blocks (6 tiles): float output, gate/up pairs for up
  // to 16 batch rows, logits for more
  const bool wide_ok = epi == EPI_F32 || (epi == EPI_SWIGLU && a.B <= 16) || (epi == EPI_LOGITS && a.B > 16);
  const bool nw_ok = epi == EPI_SWIGLU ? (a.nw == 2 || (a.nw == 6 && wide_ok)) : ((a.nw >= 1 && a.nw <= 3) || (a.nw == 6 && wide_ok));
  if (!nw_ok) SS_FAIL(SS_EINVAL, "decode GEMM: %d weight tiles per block", a.nw);
  if (a.n_blocks < 1 || a.n_blocks > units || stream_gemm_units_per_block(epi, a) * tu > a.nw)
    SS_FAIL(SS_EINVAL, "decode GEMM: %d blocks of at most %d tiles do not cover %d tiles", a.n_blocks, a.nw, a.row_tiles);
  if (a.u_base != units / a.n_blocks || a.u_rem != units % a.n_blocks || a.k_slice != ceil_div(a.k_blocks, a.k_split > 1 ? a.k_split : 1))
    SS_FAIL(SS_EINVAL, "decode GEMM: the shares (%d units, %d more for the first %d blocks, %d k blocks a slice) do not fit the shape",
            a.u_base, 1, a.u_rem, a.k_slice);
  if (!a.w || !a.act || !a.zero_frag) SS_FAIL(SS_EINVAL, "decode GEMM: NULL operand");
  if (a.k_split != 0 && a.k_split != 1 &&
      !(a.k_split >= 2 && a.k_split <= 8 && epi == EPI_F32 && a.k_blocks >= a.k_split * a.ks &&
        a.part_stride >= (size_t)a.B * a.ld_out))
    SS_FAIL(SS_EINVAL, "decode GEMM: bad split of K over blocks");
  if (epi == EPI_RESID && a.row_tiles % 2) SS_FAIL(SS_EINVAL, "decode GEMM: residual output needs whole tile pairs");
  if (a.stat_groups < 0 || (a.stat_groups > 0 && (!a.stat_in || a.norm_dim < 1 || (!a.rms && !a.wg))))
    SS_FAIL(SS_EINVAL, "decode GEMM: incomplete normalisation arguments");
  switch (epi) {
    case EPI_F32:
      if (!a.out_f32 || a.ld_out < a.N) SS_FAIL(SS_EINVAL, "decode GEMM: bad float output");
      break;
    case EPI_SWIGLU:
      if (a.row_tiles % 2 || a.N * 2 != a.row_tiles * 16) SS_FAIL(SS_EINVAL, "decode GEMM: gate/up tiles must pair up");
      // fall through
    case EPI_ACT:
      if (!a.act_out || a.N % 16 || a.out_k_blocks * (dtype == SS_DTYPE_BF16 ? 32 : 16) < a.N)
        SS_FAIL(SS_EINVAL, "decode GEMM: bad activation output");
      break;
    case EPI_RESID:
      if (!a.x_in || !a.x_out || a.N != a.row_tiles * 16 || a.stat_groups != 0 || a.wg)
        SS_FAIL(SS_EINVAL, "decode GEMM: bad residual arguments");
      if (a.act_out && (!a.g_out || !a.stat_out || a.out_k_blocks * (dtype == SS_DTYPE_BF16 ? 32 : 16) < a.N))
        SS_FAIL(SS_EINVAL, "decode GEMM: bad residual operand output");
      break;
    case EPI_LOGITS:
      if (!a.am_val || !a.am_idx || (a.out_f32 && a.ld_out < a.N))
        SS_FAIL(SS_EINVAL, "decode GEMM: bad logits arguments");
      break;
    default: SS_FAIL(SS_EINVAL, "decode GEMM: unknown epilogue %d", epi);
  }
  return SS_OK;
}

// the widest instance: LDS above the static limit is asked for once per process, then at every launch
template <typename T, int NB, int KSM, int EPI>
static ss_status launch_wide(const StreamGemmArgs &a, dim3 grid, dim3 block, hipStream_t st) {
  constexpr size_t lds = sizeof(GemmShared<NB, KSM, 6>);
  if constexpr (lds > 64 * 1024) {
    static std::atomic<bool> allowed[64];  // per device
    int dev = 0;
    SS_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) SS_FAIL(SS_EINVAL, "decode GEMM: device %d", dev);
    if (!allowed[dev].load()) {
      SS_HIP(hipFuncSetAttribute((const void *)stream_gemm<T, NB, false, EPI, KSM, 6>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                 (int)lds));
      allowed[dev].store(true);
    }
    SS_LAUNCH_KERNEL((stream_gemm<T, NB, false, EPI, KSM, 6>), grid, block, lds, st, a);
  } else {
    SS_LAUNCH_KERNEL((stream_gemm<T, NB, false, EPI, KSM, 6>), grid, block, 0, st, a);
  }
  return SS_OK;
}

template <typename T, int NB, int KSM>
static ss_status launch_stream_gemm_t(int epi, const StreamGemmArgs &a, dim3 grid, dim3 block, hipStream_t st) {
#define SS_LAUNCH(GLU, EPI, NW) SS_LAUNCH_KERNEL((stream_gemm<T, NB, GLU, EPI, KSM, NW>), grid, block, 0, st, a)
  if (epi == EPI_SWIGLU) {
    if constexpr (NB == 1) {
      if (a.nw == 6) {
        SS_LAUNCH(true, EPI_SWIGLU, 6);
        return SS_OK;
      }
    }
    SS_LAUNCH(true, EPI_SWIGLU, 2);
  } else if (a.nw == 6) {  // wide blocks: float output; logits for more than 16 batch rows
    if constexpr (NB == 2) {
      if (epi == EPI_LOGITS) return launch_wide<T, NB, KSM, EPI_LOGITS>(a, grid, block, st);
    }
    return launch_wide<T, NB, KSM, EPI_F32>(a, grid, block, st);
  } else if (a.nw == 3) {
    if (epi == EPI_F32) SS_LAUNCH(false, EPI_F32, 3);
    else if (epi == EPI_ACT) SS_LAUNCH(false, EPI_ACT, 3);
    else if (epi == EPI_RESID) SS_LAUNCH(false, EPI_RESID, 3);
    else SS_LAUNCH(false, EPI_LOGITS, 3);
  } else if (a.nw == 1) {
    if (epi == EPI_F32) SS_LAUNCH(false, EPI_F32, 1);
    else if (epi == EPI_ACT) SS_LAUNCH(false, EPI_ACT, 1);
    else if (epi == EPI_RESID) SS_LAUNCH(false, EPI_RESID, 1);
    else SS_LAUNCH(false, EPI_LOGITS, 1);
  } else {
    if (epi == EPI_F32) SS_LAUNCH(false, EPI_F32, 2);
    else if (epi == EPI_ACT) SS_LAUNCH(false, EPI_ACT, 2);
    else if (epi == EPI_RESID) SS_LAUNCH(false, EPI_RESID, 2);
    else SS_LAUNCH(false, EPI_LOGITS, 2);
  }
#undef SS_LAUNCH
  return SS_OK;
}

ss_status launch_stream_gemm(int dtype, int epi, const StreamGemmArgs &a, hipStream_t st) {
  SS_TRY(check_stream_gemm(dtype, epi, a));
  const dim3 grid(a.n_blocks * (a.k_split > 1 ? a.k_split : 1)), block(a.ks * 64);
  const int nb = a.B <= 16 ? 1 : 2;
  if (dtype == SS_DTYPE_BF16) {
    if (nb == 1) SS_TRY((launch_stream_gemm_t<bf16_t, 1, 8>(epi, a, grid, block, st)));
    else SS_TRY((launch_stream_gemm_t<bf16_t, 2, 8>(epi, a, grid, block, st)));
  } else {
    if (nb == 1) SS_TRY((launch_stream_gemm_t<float, 1, 8>(epi, a, grid, block, st)));
    else SS_TRY((launch_stream_gemm_t<float, 2, 8>(epi, a, grid, block, st)));
  }
  SS_HIP(hipGetLastError());
  return SS_OK;
}

// ---------------------------------------------------------------------------
// The first FFN matrix with K cut into slices (more than 16 batch rows, where the tiles alone fill too
// few compute units and every block pays for the whole activation slab): the GEMM leaves S raw
// partial products in float32 (EPI_F32 above, without normalisation or bias: its blocks then read no row
// statistics at all, which at d = 9216 are 147 KB a block), and this kernel adds them in slice order,
// applies the deferred normalisation rstd * (sum - (mean - c) * wg[n]) + cb[n] and the activation, and
// writes the second FFN matrix's operand fragments.
// grid = (ceil(N / 1024), B): a block takes 1024 consecutive features of one batch row, a thread four;
// the row's statistics are added up by the block itself (thread t the producer's partials t, t + 256, ...;
// the threads in order of their number: a fixed order).  a.out_f32 / part_stride / ld_out / k_split
// describe the partials, a.stat_in ... a.cb the normalisation (as for the GEMMs), a.act_out /
// out_k_blocks / act_kind the output.
// ---------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) act_fixup(StreamGemmArgs a) {
  typedef typename Operand<T>::type OT;
  __shared__ float2 s_part[256];
  __shared__ float s_mean, s_rstd;
  const int tid = threadIdx.x, b = blockIdx.y;
  const int n0 = (blockIdx.x * 256 + tid) * 4;
  const bool live = n0 < a.N;
  // everything from memory is requested first: the partial products, the folded vectors, the row's partial sums
  const float *src = a.out_f32 + (size_t)b * a.ld_out + (live ? n0 : 0);
  f32x4 part[kQkvParts];
#pragma unroll
  for (int s = 0; s < kQkvParts; ++s)
    if (s < a.k_split) part[s] = *(const f32x4 *)(src + (size_t)s * a.part_stride);
  f32x4 wg = {0.f, 0.f, 0.f, 0.f}, cb = {0.f, 0.f, 0.f, 0.f};
  if (a.wg) wg = *(const f32x4 *)(a.wg + (live ? n0 : 0));
  if (a.cb) cb = *(const f32x4 *)(a.cb + (live ? n0 : 0));
  float mean = 0.f, rstd = 1.f;
  if (a.stat_groups > 0) {
    f32x4 sv = {0.f, 0.f, 0.f, 0.f};
    for (int g = tid; g < a.stat_groups; g += 256) sv += ((const f32x4 *)a.stat_in)[(size_t)g * 32 + b];
    s_part[tid] = make_float2(sv[0] + sv[2], sv[1] + sv[3]);
    __syncthreads();
    if (tid < 64) {  // one wave: 4 partials a lane in order, then the lanes by a butterfly (a fixed order)
      float u1 = 0.f, u2 = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) u1 += s_part[tid * 4 + i].x, u2 += s_part[tid * 4 + i].y;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) u1 += __shfl_xor(u1, off), u2 += __shfl_xor(u2, off);
      if (tid == 0) {
        const float inv = 1.0f / (float)a.norm_dim;
        const float ms = u2 * inv;
        float m = 0.f, r;
        if (a.rms) {
          r = rsqrtf(ms + a.eps);
        } else {
          m = u1 * inv;
          r = rsqrtf(fmaxf(ms - m * m, 0.f) + a.eps);
          // the next producer centres on this norm's mean (one block per row)
          if (a.publish && a.cen && blockIdx.x == 0) a.cen[b] = a.cen[b] + m;
        }
        s_mean = m, s_rstd = r;
      }
    }
    __syncthreads();
    mean = s_mean, rstd = s_rstd;
  }
  if (!live) return;
  f32x4 h = part[0];
#pragma unroll
  for (int s = 1; s < kQkvParts; ++s)
    if (s < a.k_split) h += part[s];
  float u[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) u[i] = act_apply(a.act_kind, rstd * (h[i] - mean * wg[i]) + cb[i]);
  store4_frag<OT, false>(a.act_out, b, n0, a.out_k_blocks, u);
}

ss_status check_act_fixup(int dtype, const StreamGemmArgs &a) {
  if (dtype != SS_DTYPE_BF16 && dtype != SS_DTYPE_F32) SS_FAIL(SS_EINVAL, "activation of the sliced FFN GEMM: dtype %d", dtype);
  if (a.B < 1 || a.B > 32 || a.N < 16 || a.N % 16 || a.ld_out < a.N || a.ld_out % 4)
    SS_FAIL(SS_EINVAL, "activation of the sliced FFN GEMM: bad shape (batch %d, N %d, row length %d)", a.B, a.N, a.ld_out);
  if (a.k_split < 2 || a.k_split > kQkvParts || a.part_stride < (size_t)a.B * a.ld_out || a.part_stride % 4)
    SS_FAIL(SS_EINVAL, "activation of the sliced FFN GEMM: %d slices, %zu floats apart", a.k_split, a.part_stride);
  if (!a.out_f32 || !a.act_out || a.out_k_blocks * (dtype == SS_DTYPE_BF16 ? 32 : 16) < a.N)
    SS_FAIL(SS_EINVAL, "activation of the sliced FFN GEMM: bad buffers");
  if (a.stat_groups < 0 || (a.stat_groups > 0 && (!a.stat_in || a.norm_dim < 1 || (!a.rms && !a.wg))))
    SS_FAIL(SS_EINVAL, "activation of the sliced FFN GEMM: incomplete normalisation arguments");
  if (a.act_kind != SS_ACT_GELU_TANH && a.act_kind != SS_ACT_RELU) SS_FAIL(SS_EINVAL, "activation of the sliced FFN GEMM: kind %d", a.act_kind);
  return SS_OK;
}

int act_fixup_blocks(const StreamGemmArgs &a) { return ceil_div(a.N, 1024); }  // per batch row

ss_status launch_act_fixup(int dtype, const StreamGemmArgs &a, hipStream_t st) {
  SS_TRY(check_act_fixup(dtype, a));
  const dim3 grid(act_fixup_blocks(a), a.B), block(256);
  if (dtype == SS_DTYPE_BF16) SS_LAUNCH_KERNEL(act_fixup<bf16_t>, grid, block, 0, st, a);
  else SS_LAUNCH_KERNEL(act_fixup<float>, grid, block, 0, st, a);
  SS_HIP(hipGetLastError());
  return SS_OK;
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
