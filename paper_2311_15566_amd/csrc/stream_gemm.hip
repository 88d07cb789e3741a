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

// grid = tile pairs, block = a.ks waves.  Wave s streams k blocks [s * per, (s + 1) * per) of
// both tiles in register batches of U fragments per tile, two batches in flight.
// KSM: waves per block at most
template <typename T, int NB, bool GLU, int EPI, int KSM, int NW>
__global__ void __launch_bounds__(KSM * 64, 2) stream_gemm(StreamGemmArgs a) {
  typedef typename Operand<T>::type OT;  // element type of the activation operands
  constexpr bool H16 = sizeof(T) == 2;     // bf16 models: weight fragments are stored as halves
  constexpr int RB = NB * 16;
  constexpr int NEP = GLU ? NB : NW * NB;  // waves that run the epilogue
  constexpr int NWE = GLU ? 2 : 1;         // weight tiles one epilogue wave combines
  __shared__ GemmShared<NB, KSM, NW> sh;
  const int tid = threadIdx.x, lane = tid & 63, ks = tid >> 6, KS = blockDim.x >> 6;
  // Block -> (tile-pair block, batch tile).  With a.bt_split == 2 (more than 16 batch rows, NB == 1)
  // the two 16-row batch tiles of a tile pair go to two blocks; workgroups go to the 8 XCDs
  // round-robin, so the two are numbered 8 apart: same XCD, same L2, the weights come from HBM once.
  int blk = blockIdx.x, bt = 0;
  if (a.bt_split == 2) {
    const int pid = blockIdx.x, nfull = (a.n_blocks / 8) * 16;
    if (pid < nfull) {
      blk = (pid / 16) * 8 + (pid % 8), bt = (pid % 16) / 8;
    } else {
      blk = (a.n_blocks / 8) * 8 + (pid - nfull) / 2, bt = (pid - nfull) % 2;
    }
  }
  // EPI_F32 with a.k_split == 2: two blocks per tile group, each over half of K; they leave two
  // partial outputs (out_f32 and out_f32 + part_stride) that the consumer adds up, so neither
  // waits for the other.  The second half contributes acc * rstd only (no mean, no bias).
  int kh = 0;
  if (EPI == EPI_F32 && a.k_split == 2) kh = blk & 1, blk >>= 1;
  const int row0 = bt * 16;       // first batch row of this block
  const int tile0 = blk * NW;
  const int k_half = (EPI == EPI_F32 && a.k_split == 2) ? (a.k_blocks + 1) / 2 : a.k_blocks;
  const int k_lo = kh * k_half, k_hi = min(a.k_blocks, k_lo + k_half);
  const int per = (k_hi - k_lo + KS - 1) / KS;
  const int k0 = k_lo + ks * per, k1 = min(k_hi, k0 + per);
  const int r = lane & 15, q4 = (lane >> 4) * 4;

  bool tile_ok[NW];
  const u32x4 *wp[NW];
#pragma unroll
  for (int j = 0; j < NW; ++j) {
    tile_ok[j] = tile0 + j < a.row_tiles;
    wp[j] = (const u32x4 *)a.w + (size_t)(tile0 + j) * a.k_blocks * 64 + lane;
  }
  bool row_ok[NB];
  const u32x4 *ap[NB];
#pragma unroll
  for (int t = 0; t < NB; ++t) {
    row_ok[t] = row0 + t * 16 + r < a.B;
    ap[t] = (const u32x4 *)a.act + (size_t)(bt + t) * a.k_blocks * 64 + lane;
  }

  // what the epilogue needs from memory is requested first, so that it has long arrived
  const bool is_epi = ks < NEP;
  const int je = GLU ? 0 : ks % NW, te = GLU ? ks : ks / NW;
  const int bl = te * 16 + r;                                       // this lane's batch row within the block
  const int b = row0 + bl;                                          // ... and in the batch
  const int wrow = (tile0 + je) * 16 + q4;                          // first of its four weight rows
  const int n0 = GLU ? blk * 16 + q4 : wrow;                        // first of its four outputs
  const bool tile_e_ok = tile0 + je < a.row_tiles;
  const bool epi_live = is_epi && tile_e_ok && b < a.B && n0 < a.N;
  f32x4 e_wg[NWE], e_cb[NWE], e_x = {0.f, 0.f, 0.f, 0.f}, e_g = {1.f, 1.f, 1.f, 1.f};
  float e_cen = 0.f;  // EPI_RESID: the centre of the operand it writes; a publishing consumer: the centre of the one it reads
  if (is_epi && a.cen && b < a.B && (EPI == EPI_RESID || (a.publish && blk == 0 && kh == 0))) e_cen = a.cen[b];
#pragma unroll
  for (int jj = 0; jj < NWE; ++jj) {
    e_wg[jj] = e_cb[jj] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (epi_live && kh == 0) {
      if (a.wg) e_wg[jj] = *(const f32x4 *)(a.wg + wrow + jj * 16);
      if (a.cb) e_cb[jj] = *(const f32x4 *)(a.cb + wrow + jj * 16);
    }
  }
  if (EPI == EPI_RESID && epi_live) {
    e_x = *(const f32x4 *)(a.x_in + (size_t)b * a.N + n0);
    if (a.act_out) e_g = *(const f32x4 *)(a.g_out + n0);
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
        for (int t = 0; t < NB; ++t) acc[t][j] = H16 ? mma_f16(w[j][u], av[t][u], acc[t][j]) : Mma<T>::mma(w[j][u], av[t][u], acc[t][j]);
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
  const f32x4 *st_p = (const f32x4 *)a.stat_in + row0 + st_loc;
  f32x4 st_v[NB][SR > 0 ? SR : 1];
  if (NORMED) {
#pragma unroll
    for (int t = 0; t < NB; ++t)
#pragma unroll
      for (int i = 0; i < SR; ++i) {
        const int g = st_slice + i * nsl;
        st_v[t][i] = (row0 + t * 16 + st_loc < a.B && g < a.stat_groups) ? st_p[(size_t)g * 32 + t * 16]
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
      if (row0 + t * 16 + st_loc < a.B)
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

  float bv = -INFINITY;  // EPI_LOGITS: this lane's best
  int bi = INT_MAX;
  if (is_epi) {
    f32x4 sum[NWE];
#pragma unroll
    for (int jj = 0; jj < NWE; ++jj) {
      const int j = GLU ? jj : je;
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
        // the next producer centres on this norm's mean (one lane per row, first block, first tile)
        if (a.publish && a.cen && blk == 0 && kh == 0 && je == 0 && lane < 16 && b < a.B) a.cen[b] = e_cen + mean;
      }
    }
    float h[NWE][4];  // the product with normalisation and bias applied
#pragma unroll
    for (int jj = 0; jj < NWE; ++jj)
#pragma unroll
      for (int i = 0; i < 4; ++i) h[jj][i] = rstd * (sum[jj][i] - mean * e_wg[jj][i]) + e_cb[jj][i];

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
        for (int i = 0; i < 4; ++i) u[i] = GLU ? silu_f(h[0][i]) * h[NWE - 1][i] : act_apply(a.act_kind, h[0][i]);
        store4_frag<OT, false>(a.act_out, b, n0, a.out_k_blocks, u);
      }
    } else if (EPI == EPI_RESID) {
      float s1 = 0.f, s2 = 0.f;
      if (epi_live) {
        float v[4], g[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          v[i] = e_x[i] + h[0][i];
          const float t = v[i] - e_cen;
          s1 += t, s2 += t * t;
          g[i] = t * e_g[i];
        }
        *(f32x4 *)(a.x_out + (size_t)b * a.N + n0) = f32x4{v[0], v[1], v[2], v[3]};
        if (a.act_out) store4_frag<OT, false>(a.act_out, b, n0, a.out_k_blocks, g);
      }
      if (a.act_out) {  // partial row sums of this weight tile's 16 features
        s1 += __shfl_xor(s1, 16), s2 += __shfl_xor(s2, 16);
        s1 += __shfl_xor(s1, 32), s2 += __shfl_xor(s2, 32);
        if (lane < 16 && tile_e_ok && b < a.B)  // tile pair blockIdx.x, half je of its float4
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
  if (tid < RB && row0 + tid < a.B) {
    bv = sh.lg_v[0][tid], bi = sh.lg_i[0][tid];
#pragma unroll
    for (int j = 1; j < NW; ++j) {
      const float ov = sh.lg_v[j][tid];
      const int oi = sh.lg_i[j][tid];
      if (ov > bv || (ov == bv && oi < bi)) bv = ov, bi = oi;
    }
    a.am_val[(size_t)(row0 + tid) * a.n_blocks + blk] = bv;   // [row][block]: a row's candidates are contiguous
    a.am_idx[(size_t)(row0 + tid) * a.n_blocks + blk] = bi;
  }
}

int stream_gemm_blocks(int epi, const StreamGemmArgs &a) {
  return ceil_div(a.row_tiles, epi == EPI_SWIGLU ? 2 : a.nw);
}

ss_status check_stream_gemm(int dtype, int epi, const StreamGemmArgs &a) {
  if (dtype != SS_DTYPE_BF16 && dtype != SS_DTYPE_F32) SS_FAIL(SS_EINVAL, "decode GEMM: dtype %d", dtype);
  if (a.B < 1 || a.B > 32) SS_FAIL(SS_EINVAL, "decode GEMM: batch %d", a.B);
  if (a.n_blocks != stream_gemm_blocks(epi, a) || (a.bt_split != 1 && !(a.bt_split == 2 && a.B > 16)))
    SS_FAIL(SS_EINVAL, "decode GEMM: bad block count / batch split");
  if (a.nw != 1 && a.nw != 2 && !(a.nw == 3 && (epi == EPI_F32 || epi == EPI_ACT) && a.ks == 8))
    SS_FAIL(SS_EINVAL, "decode GEMM: %d weight tiles per block", a.nw);
  if (a.row_tiles < 1 || a.k_blocks < 1 || (a.ks != 4 && a.ks != 8) || a.N < 1 || a.N > a.row_tiles * 16)
    SS_FAIL(SS_EINVAL, "decode GEMM: bad shape (tiles %d, k blocks %d, waves %d, N %d)", a.row_tiles, a.k_blocks, a.ks, a.N);
  if (!a.w || !a.act) SS_FAIL(SS_EINVAL, "decode GEMM: NULL operand");
  if (a.k_split != 0 && a.k_split != 1 &&
      !(a.k_split == 2 && epi == EPI_F32 && a.bt_split == 1 && a.k_blocks >= 2 * a.ks && a.part_stride >= (size_t)a.B * a.ld_out))
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

template <typename T, int NB, int KSM>
static void launch_stream_gemm_t(int epi, const StreamGemmArgs &a, dim3 grid, dim3 block, hipStream_t st) {
#define SS_LAUNCH(GLU, EPI, NW) SS_LAUNCH_KERNEL((stream_gemm<T, NB, GLU, EPI, KSM, NW>), grid, block, 0, st, a)
  if (epi == EPI_SWIGLU) SS_LAUNCH(true, EPI_SWIGLU, 2);
  else if (a.nw == 3) {  // q|k|v and first-FFN matrices with more tile pairs than compute units
    if (epi == EPI_F32) SS_LAUNCH(false, EPI_F32, 3);
    else SS_LAUNCH(false, EPI_ACT, 3);
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
}

ss_status launch_stream_gemm(int dtype, int epi, const StreamGemmArgs &a, hipStream_t st) {
  SS_TRY(check_stream_gemm(dtype, epi, a));
  const dim3 grid(stream_gemm_blocks(epi, a) * a.bt_split * (a.k_split == 2 ? 2 : 1)), block(a.ks * 64);
  const int nb = (a.B <= 16 || a.bt_split == 2) ? 1 : 2;
  if (dtype == SS_DTYPE_BF16) {
    if (nb == 1) launch_stream_gemm_t<bf16_t, 1, 8>(epi, a, grid, block, st);
    else launch_stream_gemm_t<bf16_t, 2, 8>(epi, a, grid, block, st);
  } else {
    if (nb == 1) launch_stream_gemm_t<float, 1, 8>(epi, a, grid, block, st);
    else launch_stream_gemm_t<float, 2, 8>(epi, a, grid, block, st);
  }
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
