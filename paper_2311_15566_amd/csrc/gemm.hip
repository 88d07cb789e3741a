// The tiled GEMM of the initial phase (matrix-core bound).
#include "kernels.h"
#include "mma.h"

#include <limits.h>
#include <math.h>
#include <stdlib.h>

#include <algorithm>

namespace ss {

// ---------------------------------------------------------------------------
// tiled prefill GEMM: block = 128 output features x 128 tokens, 4 waves of 64 x 64,
// K advanced two fragments at a time through LDS with register prefetch of the next stage.
// ---------------------------------------------------------------------------
// bf16 models: the activation operands and the stored weight fragments are halves; float32 models: floats.
template <typename T, int EPI>
__global__ void __launch_bounds__(256) tile_gemm(TileGemmArgs a) {
  constexpr bool H16 = sizeof(T) == 2;
  typedef typename Operand<T>::type OT;  // element type of the activation operands
  constexpr int KS = 2;  // k fragments per stage
  __shared__ __align__(16) u32x4 lds_w[KS][8][64];
  __shared__ __align__(16) u32x4 lds_a[KS][8][64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 1, wc = wave & 1;
  // Block -> output tile.  Workgroups go to the 8 XCDs round-robin and each XCD has its own L2, so
  // XCD x takes a contiguous run of the tile list, ordered so that the blocks running together
  // on it are a few token blocks times a window of row blocks: weight panels are shared by the
  // token blocks of a group, activation panels by the row blocks of the window.
  int rb, tb;
  {
    constexpr int GT = 8;  // token blocks per group
    const int nrb = a.n_row_blocks, ntb = a.T / 128, nblk = nrb * ntb;
    const int pid = blockIdx.x, xcd = pid % 8, local = pid / 8;
    const int base = nblk / 8, rem = nblk % 8;
    const int L = xcd * base + min(xcd, rem) + local;
    const int group = L / (GT * nrb), first_tb = group * GT;
    const int gsz = min(GT, ntb - first_tb), within = L - group * GT * nrb;
    tb = first_tb + within % gsz;
    rb = within / gsz;
  }
  const int rt0 = rb * 8;   // first weight row tile
  const int tt0 = tb * 8;   // first token tile
  const u32x4 *W = (const u32x4 *)a.w;
  const u32x4 *A = (const u32x4 *)a.act;

  f32x4 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // per stage each thread moves 4 weight pieces and 4 activation pieces:
  // piece p = tid + 256*r -> (ks = p / 512, tile = (p / 64) % 8, ln = p % 64)
  u32x4 pw[4], pa[4];
  auto fetch = [&](int kb) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int p = tid + 256 * r;
      const int ks = p >> 9, tile = (p >> 6) & 7, ln = p & 63;
      const int k = kb + ks;
      const bool kok = k < a.k_blocks;
      pw[r] = (kok && rt0 + tile < a.row_tiles) ? W[((size_t)(rt0 + tile) * a.k_blocks + k) * 64 + ln]
                                               : u32x4{0u, 0u, 0u, 0u};
      pa[r] = kok ? A[((size_t)(tt0 + tile) * a.k_blocks + k) * 64 + ln] : u32x4{0u, 0u, 0u, 0u};
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
      lds_a[ks][tile][ln] = pa[r];
    }
    __syncthreads();
    if (kb + KS < a.k_blocks) fetch(kb + KS);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      u32x4 wf[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) wf[i] = lds_w[ks][wr * 4 + i][lane];
      u32x4 af[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) af[j] = lds_a[ks][wc * 4 + j][lane];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = H16 ? mma_f16(wf[i], af[j], acc[i][j]) : Mma<T>::mma(wf[i], af[j], acc[i][j]);
    }
  }

  const int q4 = (lane >> 4) * 4, tl = lane & 15;
  const float *cbp = a.mr_in ? a.cb : a.bias;
  const float *wgp = a.mr_in ? a.wg : nullptr;
  // the product of weight row n0 + e and this lane's token, with the deferred norm and the bias applied
  auto finish = [&](const f32x4 &c, const int n0, const float2 mr, float (&v)[4]) {  // mr = (mean - centre, rstd)
    f32x4 wg = {0.f, 0.f, 0.f, 0.f}, cb = {0.f, 0.f, 0.f, 0.f};
    if (wgp) wg = *(const f32x4 *)(wgp + n0);
    if (cbp) cb = *(const f32x4 *)(cbp + n0);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = mr.y * (c[e] - mr.x * wg[e]) + cb[e];
  };
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int tok = (tt0 + wc * 4 + j) * 16 + tl;
    const bool tok_live = tok < a.T_live;
    if (EPI == EPI_SWIGLU) {
      const float2 mr = a.mr_in ? make_float2(a.mr_in[tok][2], a.mr_in[tok][1]) : make_float2(0.f, 1.f);
#pragma unroll
      for (int i = 0; i < 4; i += 2) {
        const int rt = rt0 + wr * 4 + i;  // gate tile; rt + 1 is the matching up tile
        const int n0 = (rt >> 1) * 16 + q4;
        if (tok_live && rt + 1 < a.row_tiles && n0 < a.N) {
          float gt[4], up[4], u[4];
          finish(acc[i][j], rt * 16 + q4, mr, gt);
          finish(acc[i + 1][j], (rt + 1) * 16 + q4, mr, up);
#pragma unroll
          for (int e = 0; e < 4; ++e) u[e] = silu_f(gt[e]) * up[e];
          store4_frag<OT, false>(a.act_out, tok, n0, a.out_k_blocks, u);
        }
      }
    } else if (EPI == EPI_RESID) {
      float s1 = 0.f, s2 = 0.f;
      const float cen = a.g_out ? a.c_in[tok][0] : 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int rt = rt0 + wr * 4 + i;
        const int n0 = rt * 16 + q4;
        if (tok_live && rt < a.row_tiles && n0 < a.N) {
          f32x4 *xp = (f32x4 *)(a.x_resid + (size_t)tok * a.N + n0);
          const f32x4 x = *xp;
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = x[e] + (acc[i][j][e] + (a.bias ? a.bias[n0 + e] : 0.f));
          *xp = f32x4{v[0], v[1], v[2], v[3]};
          if (a.g_out) {
            const f32x4 g = *(const f32x4 *)(a.g_out + n0);
            float y[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float t = v[e] - cen;
              s1 += t, s2 += t * t;
              y[e] = t * g[e];
            }
            store4_frag<OT, false>(a.norm_out, tok, n0, a.N / Elem<OT>::kFragK, y);
          }
        }
      }
      if (a.g_out) {  // the wave's 64 features of this token
        s1 += __shfl_xor(s1, 16), s2 += __shfl_xor(s2, 16);
        s1 += __shfl_xor(s1, 32), s2 += __shfl_xor(s2, 32);
        if (lane < 16) a.stat_out[(size_t)(rb * 2 + wr) * a.T + tok] = make_float2(s1, s2);
      }
    } else {
      const float2 mr = a.mr_in ? make_float2(a.mr_in[tok][2], a.mr_in[tok][1]) : make_float2(0.f, 1.f);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int rt = rt0 + wr * 4 + i;
        const int n0 = rt * 16 + q4;
        if (tok_live && rt < a.row_tiles && n0 < a.N) {
          float v[4];
          finish(acc[i][j], n0, mr, v);
          if (EPI == EPI_F32) {
            *(f32x4 *)(a.out_f32 + (size_t)tok * a.ld_out + n0) = f32x4{v[0], v[1], v[2], v[3]};
          } else {  // EPI_ACT
            const float w[4] = {act_apply(a.act_kind, v[0]), act_apply(a.act_kind, v[1]), act_apply(a.act_kind, v[2]),
                                act_apply(a.act_kind, v[3])};
            store4_frag<OT, false>(a.act_out, tok, n0, a.out_k_blocks, w);
          }
        }
      }
    }
  }
}

__global__ void __launch_bounds__(256) row_stats(const float2 *part, int groups, int T, float inv_dim, int rms, float eps,
                                                 f32x4 *mr) {
  const int tok = blockIdx.x * 256 + threadIdx.x;
  if (tok >= T) return;
  const float c = mr[tok][0];  // the centre the partial sums were taken about
  float u1 = 0.f, u2 = 0.f;
  int g = 0;
  for (; g + 8 <= groups; g += 8) {  // eight loads in flight; the sums stay in group order
    float2 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = part[(size_t)(g + i) * T + tok];
#pragma unroll
    for (int i = 0; i < 8; ++i) u1 += v[i].x, u2 += v[i].y;
  }
  for (; g < groups; ++g) {
    const float2 v = part[(size_t)g * T + tok];
    u1 += v.x, u2 += v.y;
  }
  const float ms = u2 * inv_dim;
  if (rms) {  // c = 0
    mr[tok] = f32x4{0.f, rsqrtf(ms + eps), 0.f, 0.f};
  } else {
    const float delta = u1 * inv_dim;  // mean - c
    mr[tok] = f32x4{c + delta, rsqrtf(fmaxf(ms - delta * delta, 0.f) + eps), delta, 0.f};
  }
}

ss_status launch_row_stats(const float2 *part, int groups, int T, int norm_dim, int rms, float eps, f32x4 *mr,
                           hipStream_t st) {
  if (!part || !mr || groups < 1 || T < 1 || norm_dim < 1) SS_FAIL(SS_EINVAL, "row statistics: bad arguments");
  hipLaunchKernelGGL(row_stats, dim3(ceil_div(T, 256)), dim3(256), 0, st, part, groups, T, 1.0f / (float)norm_dim, rms, eps, mr);
  SS_HIP(hipGetLastError());
  return SS_OK;
}

ss_status launch_tile_gemm(int dtype, int epi, TileGemmArgs a, hipStream_t st) {
  if (a.T < 128 || a.T % 128) SS_FAIL(SS_EINVAL, "prefill GEMM: token count %d is not a multiple of 128", a.T);
  if (a.row_tiles < 1 || a.k_blocks < 1 || a.N % 4) SS_FAIL(SS_EINVAL, "prefill GEMM: bad shape");
  if ((epi == EPI_F32 && (a.ld_out % 4)) || epi == EPI_LOGITS) SS_FAIL(SS_EINVAL, "prefill GEMM: bad epilogue");
  if (epi == EPI_RESID && a.g_out) {
    const int fk = dtype == SS_DTYPE_BF16 ? 32 : 16;
    if (!a.norm_out || !a.stat_out || !a.c_in || a.N % fk || a.N != a.row_tiles * 16)
      SS_FAIL(SS_EINVAL, "prefill GEMM: bad next-operand arguments");
  }
  a.n_row_blocks = ceil_div(a.row_tiles, 8);
  dim3 grid(a.n_row_blocks * (a.T / 128));
#define SS_LAUNCH(TT, EPI) hipLaunchKernelGGL((tile_gemm<TT, EPI>), grid, dim3(256), 0, st, a)
  if (dtype == SS_DTYPE_BF16) {
    if (epi == EPI_F32) SS_LAUNCH(bf16_t, EPI_F32);
    else if (epi == EPI_RESID) SS_LAUNCH(bf16_t, EPI_RESID);
    else if (epi == EPI_ACT) SS_LAUNCH(bf16_t, EPI_ACT);
    else SS_LAUNCH(bf16_t, EPI_SWIGLU);
  } else {
    if (epi == EPI_F32) SS_LAUNCH(float, EPI_F32);
    else if (epi == EPI_RESID) SS_LAUNCH(float, EPI_RESID);
    else if (epi == EPI_ACT) SS_LAUNCH(float, EPI_ACT);
    else SS_LAUNCH(float, EPI_SWIGLU);
  }
#undef SS_LAUNCH
  SS_HIP(hipGetLastError());
  return SS_OK;
}

}  // namespace ss
