// The tiled GEMM of the initial phase (matrix-core bound).
#include "kernels.h"
#include "mma.h"

#include <limits.h>
#include <math.h>
#include <stdlib.h>

#include <algorithm>
#include <atomic>
#include <mutex>
#include <type_traits>

namespace ss {

// ---------------------------------------------------------------------------
// tiled prefill GEMM: block = 128 output features x 128 or 256 tokens, 4 waves of 64 x 64 or 64 x 128.
// One k fragment per stage; the stages go from global memory straight into a ring of three LDS
// buffers (no registers in between): while stage k is multiplied, stage k + 1 has landed or is
// landing and stage k + 2 is requested.  Per matrix-core instruction a wave reads 3/8 of a
// fragment from LDS (1/2 with 64 x 64 wave tiles).
// ---------------------------------------------------------------------------
// s_waitcnt with only the vector-memory counter set (gfx9 encoding: vmcnt = simm16[3:0] and
// simm16[15:14]; the export and LDS counters stay at their maxima, i.e. are not waited for)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// The accumulators of a 128 x 128 wave tile fill all 256 accumulation registers and the operands must stay in the
// ordinary ones; the register allocator does not find that split by itself (it parks operands in accumulation
// registers and shuffles accumulators in and out), so the product of that tile is written with the classes spelled out.
// Written this way the compiler no longer sees a matrix-core instruction: the wait states between the last product and
// the first read of an accumulator are inserted by hand (drain_mma); between products nothing is needed, every
// accumulator being used once per 64 products and the operands written by LDS reads only (waited for by counter).
// FIRST: the product alone (added to the constant 0), which also defines the accumulator
template <bool FIRST>
__device__ __forceinline__ void mma_f16_pinned(f32x4 &c, const u32x4 &w, const u32x4 &a) {
  if constexpr (FIRST) asm("v_mfma_f32_16x16x32_f16 %0, %1, %2, 0" : "=a"(c) : "v"(w), "v"(a));
  else asm("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(c) : "v"(w), "v"(a));
}
__device__ __forceinline__ void drain_mma() {
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
}

// bf16 models: the activation operands and the stored weight fragments are halves; float32 models: floats.
// Either way a fragment is 64 lanes x 16 bytes, so the loop is the same.
constexpr int kTileGemmRing = 3;  // LDS stages
constexpr int kBigBlockRounds = 4;  // 256-row blocks where there are at least this many per compute unit

// NJ: token tiles of a wave, 8 (block of 256 tokens) or 4 (128 tokens); MI: weight row tiles of a wave, 4 (block of 128 rows;
// two blocks per compute unit with 256 tokens, three with 128) or 8 (256 rows x 256 tokens, one block per compute unit and one
// wave per SIMD with a 128 x 128 tile: 2/3 of the LDS and L2 reads per flop of the 128 x 256 block)
template <typename T, int EPI, int NJ, int MI>
__global__ void __launch_bounds__(256, MI == 8 ? 1 : (NJ == 8 ? 2 : 3)) tile_gemm(TileGemmArgs a) {
  typedef typename Operand<T>::type OT;  // element type of the activation operands
  constexpr int BMT = 2 * MI, BTT = 2 * NJ;
  constexpr int STAGE = (BMT + BTT) * 64;  // 16-byte pieces per stage: weight fragments, then activation fragments
  constexpr int LPS = (BMT + BTT) / 4;     // loads a wave issues per stage
  extern __shared__ __align__(16) u32x4 lds[];  // kTileGemmRing stages
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 1, wc = wave & 1;
  // Block -> output tile.  Workgroups go to the 8 XCDs round-robin and each XCD has its own L2, so
  // XCD x takes a contiguous run of the tile list, ordered so that the blocks running together
  // on it are a few token blocks times a window of row blocks: weight panels are shared by the
  // token blocks of a group, activation panels by the row blocks of the window.
  int rb, tb;
  {
    constexpr int GT = 8;  // token blocks per group
    const int nrb = a.n_row_blocks, ntb = a.T / (BTT * 16), nblk = nrb * ntb;
    const int pid = blockIdx.x, xcd = pid % 8, local = pid / 8;
    const int base = nblk / 8, rem = nblk % 8;
    const int L = xcd * base + min(xcd, rem) + local;
    const int group = L / (GT * nrb), first_tb = group * GT;
    const int gsz = min(GT, ntb - first_tb), within = L - group * GT * nrb;
    tb = first_tb + within % gsz;
    rb = within / gsz;
  }
  const int rt0 = rb * BMT;   // first weight row tile
  const int tt0 = tb * BTT;   // first token tile
  const u32x4 *W = (const u32x4 *)a.w;
  const u32x4 *A = (const u32x4 *)a.act;
  // A two-part operand (block-uniform): the reduction runs twice, over the high parts and then, with the same
  // weights, over the low parts, into the same sums.
  const u32x4 *A_lo = (a.act_lo && rt0 >= a.lo_row_begin && rt0 < a.lo_row_end) ? (const u32x4 *)a.act_lo : nullptr;
  const int n_stages = A_lo ? 2 * a.k_blocks : a.k_blocks;

  f32x4 acc[MI][NJ];
  if constexpr (MI != 8) {  // (the 256-row block's first stage defines them)
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // Stage k -> buffer buf: every wave brings 2 weight and 4 activation fragments, each as one
  // 1 KiB load that the hardware writes to LDS at (wave-uniform base) + lane * 16.  Row tiles
  // past the matrix repeat the last one (in bounds; their outputs are never stored).
  auto issue = [&](int stage, int buf) {
    const bool second = stage >= a.k_blocks;
    const int k = second ? stage - a.k_blocks : stage;
    const u32x4 *Ak = second ? A_lo : A;
    u32x4 *st = lds + buf * STAGE;
#pragma unroll
    for (int r = 0; r < BMT / 4; ++r) {
      const int tile = wave + 4 * r;
      const int rt = min(rt0 + tile, a.row_tiles - 1);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(W + ((size_t)rt * a.k_blocks + k) * 64 + lane),
                                       (__attribute__((address_space(3))) void *)(st + tile * 64), 16, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < BTT / 4; ++r) {
      const int tile = wave + 4 * r;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(Ak + ((size_t)(tt0 + tile) * a.k_blocks + k) * 64 + lane),
                                       (__attribute__((address_space(3))) void *)(st + (BMT + tile) * 64), 16, 0, 0);
    }
  };
  // The operands of a stage are read from LDS one stage ahead of their use: while the matrix cores work on stage
  // k out of one set of registers, the reads of stage k + 1 into the other set are under way, so a wave's
  // matrix-core instructions follow each other without waiting for LDS.
  auto fetch = [&](u32x4(&wf)[MI], u32x4(&af)[NJ], int stage) {
    const u32x4 *st = lds + (stage % kTileGemmRing) * STAGE;
#pragma unroll
    for (int i = 0; i < MI; ++i) wf[i] = st[(wr * MI + i) * 64 + lane];
#pragma unroll
    for (int j = 0; j < NJ; ++j) af[j] = st[(BMT + wc * NJ + j) * 64 + lane];
  };
  auto multiply = [&](const u32x4(&wf)[MI], const u32x4(&af)[NJ]) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j) acc[i][j] = mma_op<T>(wf[i], af[j], acc[i][j]);
  };
  // Before stage s is read: this wave's share of it has landed (loads complete in order; the stages after it may
  // still be in flight), then the barrier says that everyone's has, and that everyone has the operands of stage
  // s - 1 in registers (LDS counter at zero), so that buffer can be refilled with stage s + 2.
  // Not __syncthreads(): its fence would also wait for the loads in flight.
  auto ready = [&](int s) {
    if (s + 1 < n_stages) wait_vmcnt<LPS>();
    else wait_vmcnt<0>();
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    if (s + 2 < n_stages) issue(s + 2, (s + 2) % kTileGemmRing);
  };
  issue(0, 0);
  if (n_stages > 1) issue(1, 1);
  ready(0);
  if constexpr (MI == 8) {
    // 256 accumulator registers leave room for one set of weight operands and two of activation operands: the
    // products go weight row tile by row tile, and a row tile's register takes the next stage's fragment as soon as its
    // products are issued; the next stage's activation fragments arrive in the other set during the first rows.
    static_assert(NJ == 8 && sizeof(T) == 2, "the 256-row block has 256 tokens and half-precision operands");
    // With one wave per SIMD nothing else fills the matrix cores while this wave does something else, so a stage's
    // other work is spread between its rows of products.  The barrier that says "stage s + 1 has landed and everyone
    // has stage s in registers" comes after the second row, when the last LDS read of the previous stage has long
    // returned; then the reads of stage s + 1 follow the rows that free their registers, and the eight loads of the
    // stage three ahead go two at a time behind rows 2 to 5.
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const u32x4 *src[LPS];  // this lane's piece of the wave's fragments at k = 0: weight tiles, then activation tiles
#pragma unroll
    for (int r = 0; r < BMT / 4; ++r) src[r] = W + (size_t)min(rt0 + wave_u + 4 * r, a.row_tiles - 1) * a.k_blocks * 64 + lane;
#pragma unroll
    for (int r = 0; r < BTT / 4; ++r) src[BMT / 4 + r] = A + (size_t)(tt0 + wave_u + 4 * r) * a.k_blocks * 64 + lane;
    const ptrdiff_t lo_delta = A_lo ? A_lo - A : 0;
    auto issue_piece = [&](int stage, int r) {  // r: 0 .. LPS - 1
      const bool second = stage >= a.k_blocks;
      const int k = second ? stage - a.k_blocks : stage;
      const ptrdiff_t off = (ptrdiff_t)k * 64 + ((second && r >= BMT / 4) ? lo_delta : 0);
      u32x4 *dst = lds + (stage % kTileGemmRing) * STAGE + (wave_u + 4 * r) * 64;  // (activation tiles follow the BMT weight tiles)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src[r] + off),
                                       (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
    };
    u32x4 wf[MI], af0[NJ], af1[NJ];
    fetch(wf, af0, 0);
    // full: stage s + 3 exists (known where the call is written: the steady loop's stages run without a branch, which
    // also lets the waits for LDS reads count reads instead of waiting for all of them)
    auto stage = [&](auto first, auto full, int s, const u32x4(&cur)[NJ], u32x4(&nxt)[NJ]) {
      constexpr bool FULL = decltype(full)::value;
      const bool more = FULL || s + 1 < n_stages, load = FULL || s + 3 < n_stages;
      const u32x4 *st = lds + ((s + 1) % kTileGemmRing) * STAGE;
      auto read_w = [&](int i) { wf[i] = st[(wr * MI + i) * 64 + lane]; };
      auto read_a = [&](int j) { nxt[j] = st[(BMT + wc * NJ + j) * 64 + lane]; };
#pragma unroll
      for (int i = 0; i < MI; ++i) {
#pragma unroll
        for (int j = 0; j < NJ; ++j) mma_f16_pinned<decltype(first)::value>(acc[i][j], wf[i], cur[j]);
        // (the reads are not conditional, so that the waits for them can count: behind the last stage they bring
        // whatever the ring's next buffer holds, into registers nobody uses again)
        if (i == 1) {
          if (more) {
            if (FULL || s + 2 < n_stages) wait_vmcnt<LPS>();
            else wait_vmcnt<0>();
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
          }
          read_a(0), read_a(1), read_w(0), read_w(1);
        } else if (i >= 2) {
          if (i <= 4) read_a(2 * i - 2), read_a(2 * i - 1);
          read_w(i);
        }
        if (load && i >= 2 && i < 2 + LPS / 2) issue_piece(s + 3, 2 * i - 4), issue_piece(s + 3, 2 * i - 3);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    const std::true_type yes;
    const std::false_type no;
    stage(yes, no, 0, af0, af1);
    int k = 1;
    for (; k + 4 < n_stages; k += 2) {
      stage(no, yes, k, af1, af0);
      stage(no, yes, k + 1, af0, af1);
    }
    for (; k < n_stages; k += 2) {
      stage(no, no, k, af1, af0);
      if (k + 1 < n_stages) stage(no, no, k + 1, af0, af1);
    }
    drain_mma();
  } else {
    u32x4 wf0[MI], af0[NJ], wf1[MI], af1[NJ];
    fetch(wf0, af0, 0);
    for (int k = 0; k < n_stages; k += 2) {
      if (k + 1 < n_stages) {
        ready(k + 1);
        fetch(wf1, af1, k + 1);
      }
      multiply(wf0, af0);
      if (k + 1 < n_stages) {
        if (k + 2 < n_stages) {
          ready(k + 2);
          fetch(wf0, af0, k + 2);
        }
        multiply(wf1, af1);
      }
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
  for (int j = 0; j < NJ; ++j) {
    const int tok = (tt0 + wc * NJ + j) * 16 + tl;
    const bool tok_live = tok < a.T_live;
    if (EPI == EPI_SWIGLU) {
      const float2 mr = a.mr_in ? make_float2(a.mr_in[tok][2], a.mr_in[tok][1]) : make_float2(0.f, 1.f);
#pragma unroll
      for (int i = 0; i < MI; i += 2) {
        const int rt = rt0 + wr * MI + i;  // gate tile; rt + 1 is the matching up tile
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
      const float cen = a.g_out ? a.c_in[tok][0] : 0.f;
#pragma unroll
      for (int band = 0; band < MI / 4; ++band) {  // 64 features: one partial sum each
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int i = band * 4; i < band * 4 + 4; ++i) {
        const int rt = rt0 + wr * MI + i;
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
            if (a.norm_out_lo) {
              float lo[4];
#pragma unroll
              for (int e = 0; e < 4; ++e) lo[e] = y[e] - Elem<OT>::to_f32(Elem<OT>::from_f32(y[e]));
              store4_frag<OT, false>(a.norm_out_lo, tok, n0, a.N / Elem<OT>::kFragK, lo);
            }
          }
        }
      }
      if (a.g_out) {  // 64 features of this token
        s1 += __shfl_xor(s1, 16), s2 += __shfl_xor(s2, 16);
        s1 += __shfl_xor(s1, 32), s2 += __shfl_xor(s2, 32);
        const int g = (rt0 + wr * MI) / 4 + band;  // bands past the last 128-row block have no slot
        if (lane < 16 && g < 2 * ((a.row_tiles + 7) / 8)) a.stat_out[(size_t)g * a.T + tok] = make_float2(s1, s2);
      }
      }
    } else {
      const float2 mr = a.mr_in ? make_float2(a.mr_in[tok][2], a.mr_in[tok][1]) : make_float2(0.f, 1.f);
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const int rt = rt0 + wr * MI + i;
        const int n0 = rt * 16 + q4;
        if (tok_live && rt < a.row_tiles && n0 < a.N) {
          float v[4];
          finish(acc[i][j], n0, mr, v);
          if (EPI == EPI_F32) {
            const f32x4 o = {v[0], v[1], v[2], v[3]};
            const int HD = a.kv_Hs * a.kv_Dh;
            if (a.k_cache && n0 >= HD) {  // a key or value piece: into the cache row of (sequence, position), not the q|k|v buffer
              const int is_v = n0 >= 2 * HD, f = n0 - (1 + is_v) * HD, hh = f / a.kv_Dh, dim = f - hh * a.kv_Dh;
              const int b = tok / a.kv_S, pos = tok - b * a.kv_S;
              char *row = (is_v ? a.v_cache : a.k_cache) + b * a.kv_row_stride + hh * a.kv_head_stride;
              const size_t e = (size_t)pos * a.kv_Dh + dim;
              if (a.kv_dtype == SS_DTYPE_F16) store4_cache<f16_t>((f16_t *)row + e, o);
              else if (a.kv_dtype == SS_DTYPE_BF16) store4_cache<bf16_t>((bf16_t *)row + e, o);
              else store4_cache<float>((float *)row + e, o);
            } else {
              *(f32x4 *)(a.out_f32 + (size_t)tok * a.ld_out + n0) = o;
            }
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

static std::atomic<int> g_forced_tok_tiles{0};  // test aid: 0 = not forced
static std::atomic<int> g_forced_row_tiles{0};

template <typename T, int EPI, int NJ, int MI>
static ss_status launch_one(const TileGemmArgs &a, dim3 grid, hipStream_t st) {
  constexpr size_t lds_bytes = (size_t)kTileGemmRing * (2 * MI + 2 * NJ) * 1024;  // 48, 72 or 96 KiB: above the 64 KiB that need no opt-in
  static std::once_flag once;
  static hipError_t attr = hipSuccess;
  std::call_once(once, [] {
    attr = hipFuncSetAttribute((const void *)tile_gemm<T, EPI, NJ, MI>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  });
  if (attr != hipSuccess) SS_FAIL(SS_EHIP, "prefill GEMM: %zu bytes of LDS refused: %s", lds_bytes, hipGetErrorString(attr));
  hipLaunchKernelGGL((tile_gemm<T, EPI, NJ, MI>), grid, dim3(256), lds_bytes, st, a);
  return SS_OK;
}

ss_status launch_tile_gemm(int dtype, int epi, TileGemmArgs a, hipStream_t st) {
  if (a.T < 256 || a.T % 256) SS_FAIL(SS_EINVAL, "prefill GEMM: token count %d is not a multiple of 256", a.T);
  if (a.row_tiles < 1 || a.k_blocks < 1 || a.N % 4) SS_FAIL(SS_EINVAL, "prefill GEMM: bad shape");
  if ((epi == EPI_F32 && (a.ld_out % 4)) || epi == EPI_LOGITS) SS_FAIL(SS_EINVAL, "prefill GEMM: bad epilogue");
  if (a.k_cache && (epi != EPI_F32 || !a.v_cache || a.kv_S < 1 || a.kv_Dh % 4 || a.N != 3 * a.kv_Hs * a.kv_Dh ||
                    (a.kv_dtype != SS_DTYPE_F16 && a.kv_dtype != SS_DTYPE_BF16 && a.kv_dtype != SS_DTYPE_F32)))
    SS_FAIL(SS_EINVAL, "prefill GEMM: bad cache arguments");
  if (a.act_lo && (epi != EPI_F32 || a.lo_row_begin < 0 || a.lo_row_begin % 8 || a.lo_row_end < a.lo_row_begin || a.lo_row_end % 8))
    SS_FAIL(SS_EINVAL, "prefill GEMM: a two-part operand goes with the float epilogue and whole row blocks");
  if (a.norm_out_lo && !(epi == EPI_RESID && a.g_out)) SS_FAIL(SS_EINVAL, "prefill GEMM: low parts without an operand output");
  if (epi == EPI_RESID && a.g_out) {
    const int fk = dtype == SS_DTYPE_BF16 ? 32 : 16;
    if (!a.norm_out || !a.stat_out || !a.c_in || a.N % fk || a.N != a.row_tiles * 16)
      SS_FAIL(SS_EINVAL, "prefill GEMM: bad next-operand arguments");
  }
  // Token block: measured on every GEMM shape of the GPT-20B, LLaMA-30B and OPT-66B shards, 256-token
  // blocks win by 3-9 % where the output has a few rounds of them (16384 tokens: fewer LDS and L2
  // reads per flop), 128-token blocks by 7-17 % on the 4096-token shapes (more blocks to spread over
  // the compute units) and by 8 % on a short reduction (1152), where a block is mostly epilogue.
  // Row block: 256 rows x 256 tokens (one wave per SIMD) where the output has several rounds of such blocks too.
  if (g_forced_tok_tiles.load()) a.tok_tiles = g_forced_tok_tiles.load(), a.wave_row_tiles = g_forced_row_tiles.load();
  if (a.tok_tiles != 4 && a.tok_tiles != 8) {
    const long blocks128 = (long)ceil_div(a.row_tiles, 8) * (a.T / 128);
    a.tok_tiles = (blocks128 >= 2048 && a.k_blocks >= 64) ? 8 : 4;
    a.wave_row_tiles = (blocks128 >= 4 * kBigBlockRounds * 256 && a.k_blocks >= 64) ? 8 : 4;
  }
  if (a.wave_row_tiles != 8 || a.tok_tiles != 8 || dtype != SS_DTYPE_BF16 || (a.act_lo && (a.lo_row_begin % 16 || a.lo_row_end % 16)))
    a.wave_row_tiles = 4;
  a.n_row_blocks = ceil_div(a.row_tiles, 2 * a.wave_row_tiles);
  dim3 grid(a.n_row_blocks * (a.T / (a.tok_tiles * 32)));
#define SS_LAUNCH(TT, EPI)                                                                                            \
  do {                                                                                                                \
    if constexpr (sizeof(TT) == 2) {                                                                                  \
      if (a.wave_row_tiles == 8) { SS_TRY((launch_one<TT, EPI, 8, 8>(a, grid, st))); break; }                         \
    }                                                                                                                 \
    if (a.tok_tiles == 8) SS_TRY((launch_one<TT, EPI, 8, 4>(a, grid, st)));                                           \
    else SS_TRY((launch_one<TT, EPI, 4, 4>(a, grid, st)));                                                            \
  } while (0)
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

extern "C" ss_status ss_debug_force_prefill_block(int32_t rows_per_block, int32_t tokens_per_block) {
  using namespace ss;
  const bool none = rows_per_block == 0 && tokens_per_block == 0;
  const bool small = rows_per_block == 128 && (tokens_per_block == 128 || tokens_per_block == 256);
  const bool big = rows_per_block == 256 && tokens_per_block == 256;
  if (!none && !small && !big) SS_FAIL(SS_EINVAL, "block of %d rows x %d tokens (0 x 0, 128 x 128, 128 x 256 or 256 x 256)", rows_per_block, tokens_per_block);
  g_forced_row_tiles.store(rows_per_block / 32);
  g_forced_tok_tiles.store(tokens_per_block / 32);
  return SS_OK;
}
