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
#include <utility>
#include <vector>

namespace ss {

// ---------------------------------------------------------------------------
// tiled prefill GEMM: block = 4 waves; 128 output features x 128 or 256 tokens (waves of 64 x 64 or 64 x 128, two or
// three blocks per compute unit), or 256 x 256 (waves of 128 x 128, one block per compute unit) for large outputs.
// One k fragment per stage; the stages go from global memory straight into a ring of three (256-row block: four) LDS
// buffers (no registers in between): while stage k is multiplied, stage k + 1 has landed or is
// landing and the stages behind it are requested.  Per matrix-core instruction a wave reads 1/2 (64 x 64), 3/8
// (64 x 128) or 1/4 (128 x 128) of a fragment from LDS.  All shapes walk k in the same order and add the row
// statistics up over the same 64-feature bands: same bits.
// ---------------------------------------------------------------------------
// s_waitcnt with only the vector-memory counter set (gfx9 encoding: vmcnt = simm16[3:0] and
// simm16[15:14]; the export and LDS counters stay at their maxima, i.e. are not waited for)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// The 256-row block's main loop is scheduled by hand, for two reasons.
// (1) The accumulators of its 128 x 128 wave tile fill all 256 accumulation registers and the operands must stay in the
// ordinary ones; the register allocator does not find that split by itself (it parks operands in accumulation registers
// and shuffles accumulators in and out), so the product is written with the register classes spelled out.
// (2) With one wave per SIMD nothing else fills the matrix cores while the wave does something else: the LDS reads and
// the loads of later stages must sit between the products, one at a time, and a product must wait only for the reads it
// needs, not for all that are under way (which is what the compiler's own wait insertion asks for).
// So products, LDS reads and their waits are volatile asm statements, which keep their order; the compiler sees neither a
// matrix-core instruction nor an LDS read in that loop and inserts no wait state or counter wait of its own there:
//  - an LDS read's destination is valid only after a wait_lds that covers it (reads return in order);
//  - between products nothing is needed: every accumulator is used once per 64 products;
//  - drain_mma() ends the loop: all reads returned, and the wait states between the last product and the first read of
//    an accumulator.
template <bool FIRST>  // FIRST: the product alone (added to the constant 0), which also defines the accumulator
__device__ __forceinline__ void mma_f16_pinned(f32x4 &c, const u32x4 &w, const u32x4 &a) {
  if constexpr (FIRST) asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, 0" : "=a"(c) : "v"(w), "v"(a));
  else asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(c) : "v"(w), "v"(a));
}
template <int OFF>  // 16 bytes per lane from LDS byte address addr + OFF
__device__ __forceinline__ void lds_read_async(u32x4 &dst, uint32_t addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
template <int N>  // until at most N LDS reads are under way
__device__ __forceinline__ void wait_lds() {
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N));
}
__device__ __forceinline__ void drain_mma() {
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_nop 15\n\ts_nop 15" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
}
template <int... Is, typename F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Is...>, F &&f) {
  (f(std::integral_constant<int, Is>()), ...);
}
template <int N, typename F>  // f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>)
__device__ __forceinline__ void static_for(F &&f) {
  static_for_impl(std::make_integer_sequence<int, N>(), f);
}
// The 256-row block's schedule: what follows product j of row i (slot i * 8 + j) beside an LDS read or the barrier:
// 0..7 = load r of the stage four ahead, 8..15 = step load r's pointer to the next k, -1 = nothing.  The sixteen of them
// take the slots from (2, 6) on that hold no LDS read, a load and its step next to each other.
constexpr int big_block_extra(int slot) {
  constexpr int at[16] = {2 * 8 + 6, 2 * 8 + 7, 3 * 8 + 5, 3 * 8 + 6, 3 * 8 + 7, 4 * 8 + 1, 4 * 8 + 2, 4 * 8 + 3,
                          4 * 8 + 4, 4 * 8 + 5, 4 * 8 + 6, 4 * 8 + 7, 5 * 8 + 1, 5 * 8 + 2, 5 * 8 + 3, 5 * 8 + 4};
  for (int n = 0; n < 16; ++n)
    if (at[n] == slot) return n % 2 == 0 ? n / 2 : 8 + n / 2;
  return -1;
}
// s_waitcnt vmcnt(8 * stages), stages 0..3 (wave-uniform)
__device__ __forceinline__ void wait_stages_in_flight(int stages) {
  if (stages >= 3) wait_vmcnt<24>();
  else if (stages == 2) wait_vmcnt<16>();
  else if (stages == 1) wait_vmcnt<8>();
  else wait_vmcnt<0>();
}

// bf16 models: the activation operands and the stored weight fragments are halves; float32 models: floats.
// Either way a fragment is 64 lanes x 16 bytes, so the loop is the same.
constexpr int kTileGemmRing = 3;  // LDS stages (128-row blocks)
constexpr int kBigBlockRing = 4;  // LDS stages of the 256-row block
constexpr int kBigBlockRounds = 2;  // 256-row blocks where there are at least this many per compute unit

// NJ: token tiles of a wave, 8 (block of 256 tokens) or 4 (128 tokens); MI: weight row tiles of a wave, 4 (block of 128 rows;
// two blocks per compute unit with 256 tokens, three with 128) or 8 (256 rows x 256 tokens, one block per compute unit and one
// wave per SIMD with a 128 x 128 tile: 2/3 of the LDS and L2 reads per flop of the 128 x 256 block)
template <typename T, int EPI, int NJ, int MI>
__global__ void __launch_bounds__(256, MI == 8 ? 1 : (NJ == 8 ? 2 : 3)) tile_gemm(TileGemmArgs a) {
  typedef typename Operand<T>::type OT;  // element type of the activation operands
  constexpr int BMT = 2 * MI, BTT = 2 * NJ;
  constexpr int STAGE = (BMT + BTT) * 64;  // 16-byte pieces per stage: weight fragments, then activation fragments
  constexpr int LPS = (BMT + BTT) / 4;     // loads a wave issues per stage
  extern __shared__ __align__(16) u32x4 lds[];  // kTileGemmRing or kBigBlockRing stages
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
  if constexpr (MI == 8) {
    // One set of weight operands and two of activation operands beside the 256 accumulators.  A stage's 64 products go
    // weight row tile by row tile; a row tile's register takes the next stage's fragment once its products are issued,
    // the next stage's activation fragments arrive in the other set.  The barrier that says "stage s + 1 has landed
    // and everyone has stage s in registers" comes after the second row, when the last LDS read of the previous stage
    // has long returned; the LDS reads of stage s + 1 and the eight loads of stage s + 4 (into the buffer stage s just
    // left) follow one by one behind the products of rows 2 to 7.
    static_assert(NJ == 8 && sizeof(T) == 2 && LPS == 8, "the 256-row block has 256 tokens and half-precision operands");
    constexpr int R = kBigBlockRing;
    constexpr uint32_t STAGE_BYTES = STAGE * 16;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    // Running pointers: this lane's piece of the fragment that each of the wave's eight loads brings next (weight tiles,
    // then activation tiles).  A load and the step of its pointer to the next k sit in different slots of the schedule.
    const u32x4 *gp[LPS];
#pragma unroll
    for (int r = 0; r < BMT / 4; ++r) gp[r] = W + (size_t)min(rt0 + wave_u + 4 * r, a.row_tiles - 1) * a.k_blocks * 64 + lane;
#pragma unroll
    for (int r = 0; r < BTT / 4; ++r) gp[BMT / 4 + r] = A + (size_t)(tt0 + wave_u + 4 * r) * a.k_blocks * 64 + lane;
    auto issue_piece = [&](int stage, int r) {  // r: 0 .. LPS - 1; stage: the one gp[r] stands at
      u32x4 *dst = lds + (stage % R) * STAGE + (wave_u + 4 * r) * 64;  // (activation tiles follow the BMT weight tiles)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)gp[r],
                                       (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
    };
    const uint64_t k_step = 1024;  // bytes from one k fragment to the next
    auto step = [&](int r) {  // (asm: the addition stays in its slot of the schedule)
      asm volatile("v_lshl_add_u64 %0, %0, 0, %1" : "+v"(gp[r]) : "s"(k_step));
    };
    // before the loads of stage k_blocks (two-part operand): the weights start over, the activations move to the low parts
    auto second_pass = [&]() {
      const ptrdiff_t back = (ptrdiff_t)a.k_blocks * 64;
#pragma unroll
      for (int r = 0; r < LPS; ++r) gp[r] += (r < BMT / 4 ? 0 : A_lo - A) - back;
    };
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)lds;
    const uint32_t w_at = lds0 + (uint32_t)((wr * MI) * 64 + lane) * 16;         // + 1024 per row tile
    const uint32_t a_at = lds0 + (uint32_t)((BMT + wc * NJ) * 64 + lane) * 16;   // + 1024 per token tile
    u32x4 wf[MI], af0[NJ], af1[NJ];
    // the first R stages are requested, stage 0 has landed for everyone, its operands are read
#pragma unroll
    for (int s = 0; s < R; ++s)
      if (s < n_stages) {
        if (s == a.k_blocks) second_pass();
#pragma unroll
        for (int r = 0; r < LPS; ++r) issue_piece(s, r), step(r);
      }
    wait_stages_in_flight(min(R, n_stages) - 1);
    asm volatile("s_barrier" ::: "memory");
    static_for<MI>([&](auto I) { lds_read_async<decltype(I)::value * 1024>(wf[decltype(I)::value], w_at); });
    static_for<NJ>([&](auto J) { lds_read_async<decltype(J)::value * 1024>(af0[decltype(J)::value], a_at); });
    wait_lds<0>();
    // full: stage s + R exists (known where the call is written: the steady loop's stages run without a branch)
    auto stage = [&](auto first, auto full, int s, const u32x4(&cur)[NJ], u32x4(&nxt)[NJ]) {
      constexpr bool FIRST = decltype(first)::value, FULL = decltype(full)::value;
      const bool more = FULL || s + 1 < n_stages, load = FULL || s + R < n_stages;
      const uint32_t buf = (uint32_t)((s + 1) % R) * STAGE_BYTES;
      const uint32_t w_rd = w_at + buf, a_rd = a_at + buf;
      // Order of the reads of stage s + 1: a0 a1 w0 w1 a2 a3 | w2 a4 a5 a6 a7 | w3 | w4 | w5 | w6 | w7 (w_i only after
      // row i).  Row 0 of the next stage needs w0 and every a_j: all but the last five reads.  (Behind the last
      // stage the reads bring whatever the ring's next buffer holds, into registers nobody uses again.)
      if (load && s + R == a.k_blocks) second_pass();
      wait_lds<5>();
      // Between two products there is room for about three other instructions (a wave issues one every four cycles,
      // a product keeps the matrix core busy for sixteen), so everything else is spread thinly: slot (i, j) is what
      // follows product j of row i.
      static_for<MI * NJ>([&](auto IJ) {
        constexpr int i = decltype(IJ)::value / NJ, j = decltype(IJ)::value % NJ;
        mma_f16_pinned<FIRST>(acc[i][j], wf[i], cur[j]);
        if constexpr (i == 1 && j == NJ - 1) {
          if (more) {  // block-uniform
            if constexpr (FULL) wait_vmcnt<(R - 2) * LPS>();
            else wait_stages_in_flight(min(n_stages - 2 - s, R - 2));
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
          } else {
            wait_lds<0>();
          }
        }
        // LDS reads of stage s + 1
        if constexpr (i == 2 && j == 0) lds_read_async<0 * 1024>(nxt[0], a_rd);
        if constexpr (i == 2 && j == 1) lds_read_async<1 * 1024>(nxt[1], a_rd);
        if constexpr (i == 2 && j == 2) lds_read_async<0 * 1024>(wf[0], w_rd);
        if constexpr (i == 2 && j == 3) lds_read_async<1 * 1024>(wf[1], w_rd);
        if constexpr (i == 2 && j == 4) lds_read_async<2 * 1024>(nxt[2], a_rd);
        if constexpr (i == 2 && j == 5) lds_read_async<3 * 1024>(nxt[3], a_rd);
        if constexpr (i == 3 && j == 0) lds_read_async<2 * 1024>(wf[2], w_rd);
        if constexpr (i == 3 && j == 1) lds_read_async<4 * 1024>(nxt[4], a_rd);
        if constexpr (i == 3 && j == 2) lds_read_async<5 * 1024>(nxt[5], a_rd);
        if constexpr (i == 3 && j == 3) lds_read_async<6 * 1024>(nxt[6], a_rd);
        if constexpr (i == 3 && j == 4) lds_read_async<7 * 1024>(nxt[7], a_rd);
        if constexpr (i >= 4 && j == 0) lds_read_async<(i - 1) * 1024>(wf[i - 1], w_rd);
        if constexpr (i == MI - 1 && j == NJ - 1) lds_read_async<(MI - 1) * 1024>(wf[MI - 1], w_rd);
        // the loads of stage s + R, and the steps of their pointers, one per slot
        constexpr int x = big_block_extra(i * NJ + j);
        if constexpr (x >= 0) {
          if (load) {
            if constexpr (x < LPS) issue_piece(s + R, x);
            else step(x - LPS);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      });
    };
    const std::true_type yes;
    const std::false_type no;
    stage(yes, no, 0, af0, af1);
    int k = 1;
    for (; k + 1 + R < n_stages; k += 2) {
      stage(no, yes, k, af1, af0);
      stage(no, yes, k + 1, af0, af1);
    }
    for (; k < n_stages; k += 2) {
      stage(no, no, k, af1, af0);
      if (k + 1 < n_stages) stage(no, no, k + 1, af0, af1);
    }
    drain_mma();
  } else {
    issue(0, 0);
    if (n_stages > 1) issue(1, 1);
    ready(0);
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

  // The epilogue.  Every global load it needs is issued before the first store, unconditionally and from clamped (valid)
  // addresses, so that a wave waits for memory a few times and not once per tile: with one wave per SIMD nothing else
  // covers such a wait.  Only the stores are predicated (tokens past T_live, rows past the matrix).
  const int q4 = (lane >> 4) * 4, tl = lane & 15;
  const int rtw = rt0 + wr * MI;  // the wave's first weight row tile
  auto tok_of = [&](int j) { return (tt0 + wc * NJ + j) * 16 + tl; };
  // first of this lane's four weight rows in row tile i, clamped into the per-row vectors (wg, cb, bias, gamma: N entries,
  // gate/up interleaved: row_tiles * 16)
  auto row_of = [&](int i) {
    return EPI == EPI_SWIGLU ? min(rtw + i, a.row_tiles - 1) * 16 + q4 : min((rtw + i) * 16 + q4, a.N - 4);
  };
  const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
  if constexpr (EPI == EPI_RESID) {
    constexpr int JB = 1, NB = NJ / JB;  // the tiles of x come JB token tiles at a time, one batch ahead of its use
    f32x4 bv[MI], gv[MI];
    float cen[NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      bv[i] = a.bias ? *(const f32x4 *)(a.bias + row_of(i)) : zero4;
      gv[i] = a.g_out ? *(const f32x4 *)(a.g_out + row_of(i)) : zero4;
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) cen[j] = a.g_out ? a.c_in[tok_of(j)][0] : 0.f;
    f32x4 xb[2][JB][MI];
    constexpr int SB = MI == 8 ? 1 : 4;  // token tiles whose partial sums are exchanged together (what the registers hold)
    float s1v[SB][MI / 4], s2v[SB][MI / 4];  // this lane's share of the partial sums: token tile j, band of 64 features
    auto load_x = [&](f32x4(&dst)[JB][MI], int j0) {
#pragma unroll
      for (int jj = 0; jj < JB; ++jj)
#pragma unroll
        for (int i = 0; i < MI; ++i)
          dst[jj][i] = *(const f32x4 *)(a.x_resid + (size_t)tok_of(j0 + jj) * a.N + row_of(i));
    };
    auto finish_x = [&](const f32x4(&xs)[JB][MI], int j0) {
#pragma unroll
      for (int jj = 0; jj < JB; ++jj) {
        const int j = j0 + jj, tok = tok_of(j);
        const bool tok_live = tok < a.T_live;
#pragma unroll
        for (int band = 0; band < MI / 4; ++band) {  // 64 features: one partial sum each
          float s1 = 0.f, s2 = 0.f;
#pragma unroll
          for (int i = band * 4; i < band * 4 + 4; ++i) {
            const int rt = rtw + i, n0 = rt * 16 + q4;
            if (tok_live && rt < a.row_tiles && n0 < a.N) {
              float v[4];
#pragma unroll
              for (int e = 0; e < 4; ++e) v[e] = xs[jj][i][e] + (acc[i][j][e] + bv[i][e]);
              *(f32x4 *)(a.x_resid + (size_t)tok * a.N + n0) = f32x4{v[0], v[1], v[2], v[3]};
              if (a.g_out) {
                float y[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  const float t = v[e] - cen[j];
                  s1 += t, s2 += t * t;
                  y[e] = t * gv[i][e];
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
          s1v[j % SB][band] = s1, s2v[j % SB][band] = s2;
        }
      }
    };
    constexpr bool AHEAD = !(MI == 4 && NJ == 4);  // (three blocks per compute unit: their registers do not hold a second batch)
    load_x(xb[0], 0);
#pragma unroll
    for (int jb = 0; jb < NB; ++jb) {
      if (AHEAD && jb + 1 < NB) load_x(xb[(jb + 1) & 1], (jb + 1) * JB);
      finish_x(xb[AHEAD ? (jb & 1) : 0], jb * JB);
      if (!AHEAD && jb + 1 < NB) load_x(xb[0], (jb + 1) * JB);
      static_assert(JB == 1 && NJ % SB == 0, "the exchange below takes token tiles SB at a time");
      if (a.g_out && jb % SB == SB - 1) {  // the four lanes of a token add up, the exchanges of SB token tiles under way together
#pragma unroll
        for (int jj = 0; jj < SB; ++jj)
#pragma unroll
          for (int band = 0; band < MI / 4; ++band) {
            float s1 = s1v[jj][band], s2 = s2v[jj][band];
            s1 += __shfl_xor(s1, 16), s2 += __shfl_xor(s2, 16);
            s1 += __shfl_xor(s1, 32), s2 += __shfl_xor(s2, 32);
            const int g = rtw / 4 + band;  // bands past the last 128-row block have no slot
            if (lane < 16 && g < 2 * ((a.row_tiles + 7) / 8)) a.stat_out[(size_t)g * a.T + tok_of(jb - (SB - 1) + jj)] = make_float2(s1, s2);
          }
      }
    }
  } else {
    // deferred norm and bias: rstd * (acc - (mean - centre) * wg[n]) + cb[n]
    const float *cbp = a.mr_in ? a.cb : a.bias;
    f32x4 wgv[MI], cbv[MI];
    float2 mrv[NJ];  // (mean - centre, rstd)
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      wgv[i] = a.mr_in && a.wg ? *(const f32x4 *)(a.wg + row_of(i)) : zero4;
      cbv[i] = cbp ? *(const f32x4 *)(cbp + row_of(i)) : zero4;
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      if (a.mr_in) {
        const f32x4 m = a.mr_in[tok_of(j)];
        mrv[j] = make_float2(m[2], m[1]);
      } else {
        mrv[j] = make_float2(0.f, 1.f);
      }
    }
    auto finish = [&](int i, int j, float(&v)[4]) {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = mrv[j].y * (acc[i][j][e] - mrv[j].x * wgv[i][e]) + cbv[i][e];
    };
    if constexpr (EPI == EPI_F32) {
      if (a.rope) {
        // q|k|v of a model with rotary positions: the wave holds whole heads, row tile i (low half of a head) and row
        // tile i + half_tiles (high half) pair up in the same lane.  q is rotated and stored, k rotated and written
        // to the cache, v written to the cache.  The (cos, sin) of a token tile's pairs are loaded one tile ahead.
        auto rotary = [&](auto half_tiles) {
          constexpr int HT2 = decltype(half_tiles)::value;  // row tiles per half head
          constexpr int NLO = MI / 2;                       // low-half tiles of the wave
          auto lo_tile = [&](int n) { return (n / HT2) * 2 * HT2 + n % HT2; };
          const int HD = a.kv_Hs * a.kv_Dh, HALF = a.kv_Dh / 2;
          f32x4 cs[2][NLO][2];  // [buffer][low tile][first two pairs, last two pairs] as (cos, sin, cos, sin)
          auto load_cs = [&](f32x4(&dst)[NLO][2], int j) {
            const int tok = tok_of(j), pos = tok - (tok / a.kv_S) * a.kv_S;
#pragma unroll
            for (int n = 0; n < NLO; ++n) {
              const int n0 = min((rtw + lo_tile(n)) * 16 + q4, a.N - 4), f = n0 % HD, dim = (f % a.kv_Dh) % HALF;
              const f32x4 *p = (const f32x4 *)(a.rope + (size_t)pos * HALF + dim);
              dst[n][0] = p[0], dst[n][1] = p[1];
            }
          };
          constexpr bool AHEAD = !(MI == 4 && NJ == 4);  // (three blocks per compute unit: no registers for a second set)
          load_cs(cs[0], 0);
#pragma unroll
          for (int j = 0; j < NJ; ++j) {
            if (AHEAD && j + 1 < NJ) load_cs(cs[(j + 1) & 1], j + 1);
            if (!AHEAD && j > 0) load_cs(cs[0], j);
            const int tok = tok_of(j);
            const bool tok_live = tok < a.T_live;
            const int b = tok / a.kv_S, pos = tok - b * a.kv_S;
#pragma unroll
            for (int n = 0; n < NLO; ++n) {
              const int i = lo_tile(n), rt = rtw + i, n0 = rt * 16 + q4;
              if (tok_live && rt + HT2 < a.row_tiles && n0 + HT2 * 16 < a.N) {
                float lo[4], hi[4];
                finish(i, j, lo);
                finish(i + HT2, j, hi);
                const int part = n0 / HD, f = n0 - part * HD, hh = f / a.kv_Dh, dim = f - hh * a.kv_Dh;  // part: 0 q, 1 k, 2 v
                if (part < 2) {
                  const f32x4 c01 = cs[AHEAD ? (j & 1) : 0][n][0], c23 = cs[AHEAD ? (j & 1) : 0][n][1];
                  rope_rotate(lo[0], hi[0], make_float2(c01[0], c01[1]), lo[0], hi[0]);
                  rope_rotate(lo[1], hi[1], make_float2(c01[2], c01[3]), lo[1], hi[1]);
                  rope_rotate(lo[2], hi[2], make_float2(c23[0], c23[1]), lo[2], hi[2]);
                  rope_rotate(lo[3], hi[3], make_float2(c23[2], c23[3]), lo[3], hi[3]);
                }
                const f32x4 olo = {lo[0], lo[1], lo[2], lo[3]}, ohi = {hi[0], hi[1], hi[2], hi[3]};
                if (part == 0) {
                  float *q = a.out_f32 + (size_t)tok * a.ld_out + n0;
                  *(f32x4 *)q = olo;
                  *(f32x4 *)(q + HALF) = ohi;
                } else {
                  char *row = (part == 2 ? a.v_cache : a.k_cache) + b * a.kv_row_stride + hh * a.kv_head_stride;
                  const size_t e = (size_t)pos * a.kv_Dh + dim;
                  if (a.kv_dtype == SS_DTYPE_F16) store4_cache<f16_t>((f16_t *)row + e, olo), store4_cache<f16_t>((f16_t *)row + e + HALF, ohi);
                  else if (a.kv_dtype == SS_DTYPE_BF16) store4_cache<bf16_t>((bf16_t *)row + e, olo), store4_cache<bf16_t>((bf16_t *)row + e + HALF, ohi);
                  else store4_cache<float>((float *)row + e, olo), store4_cache<float>((float *)row + e + HALF, ohi);
                }
              }
            }
          }
        };
        if (a.kv_Dh == 128) {
          if constexpr (MI == 8) rotary(std::integral_constant<int, 4>());
        } else {
          rotary(std::integral_constant<int, 2>());
        }
        return;
      }
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int tok = tok_of(j);
      const bool tok_live = tok < a.T_live;
      if constexpr (EPI == EPI_SWIGLU) {
#pragma unroll
        for (int i = 0; i < MI; i += 2) {
          const int rt = rtw + i;  // gate tile; rt + 1 is the matching up tile
          const int n0 = (rt >> 1) * 16 + q4;
          if (tok_live && rt + 1 < a.row_tiles && n0 < a.N) {
            float gt[4], up[4], u[4];
            finish(i, j, gt);
            finish(i + 1, j, up);
#pragma unroll
            for (int e = 0; e < 4; ++e) u[e] = silu_rcp(gt[e]) * up[e];
            store4_frag<OT, false>(a.act_out, tok, n0, a.out_k_blocks, u);
          }
        }
      } else {
#pragma unroll
        for (int i = 0; i < MI; ++i) {
          const int rt = rtw + i, n0 = rt * 16 + q4;
          if (tok_live && rt < a.row_tiles && n0 < a.N) {
            float v[4];
            finish(i, j, v);
            if constexpr (EPI == EPI_F32) {
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
  constexpr size_t lds_bytes = (size_t)(MI == 8 ? kBigBlockRing : kTileGemmRing) * (2 * MI + 2 * NJ) * 1024;  // 48, 72 or 128 KiB: above the 64 KiB that need no opt-in
  static std::once_flag once;
  static hipError_t attr = hipSuccess;
  std::call_once(once, [] {
    attr = hipFuncSetAttribute((const void *)tile_gemm<T, EPI, NJ, MI>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  });
  if (attr != hipSuccess) SS_FAIL(SS_EHIP, "prefill GEMM: %zu bytes of LDS refused: %s", lds_bytes, hipGetErrorString(attr));
  hipLaunchKernelGGL((tile_gemm<T, EPI, NJ, MI>), grid, dim3(256), lds_bytes, st, a);
  return SS_OK;
}

// Sets a.tok_tiles and a.wave_row_tiles.
// Token block: measured on every GEMM shape of the GPT-20B, LLaMA-30B and OPT-66B shards, 256-token
// blocks win by 3-9 % where the output has a few rounds of them (16384 tokens: fewer LDS and L2
// reads per flop), 128-token blocks by 7-17 % on the 4096-token shapes (more blocks to spread over
// the compute units).  A short reduction (OPT-66B shard's out-projection, 1152 = 36 k fragments), where a block is mostly
// epilogue, took the small block by 8 % until the epilogues issued their loads up front; now 630 us (128 x 128),
// 600 (128 x 256), 585 (256 x 256).
// Row block: 256 rows x 256 tokens (one wave per SIMD) where the output has a few rounds of such blocks too: 12-17 % faster
// than 128 x 256 on the LLaMA-30B shard's matrices, 10 % on the OPT-66B shard's.
static void choose_block(int dtype, TileGemmArgs &a) {
  if (g_forced_tok_tiles.load()) a.tok_tiles = g_forced_tok_tiles.load(), a.wave_row_tiles = g_forced_row_tiles.load();
  if (a.tok_tiles != 4 && a.tok_tiles != 8) {
    const long blocks128 = (long)ceil_div(a.row_tiles, 8) * (a.T / 128);
    a.tok_tiles = (blocks128 >= 2048 && a.k_blocks >= 32) ? 8 : 4;
    a.wave_row_tiles = (blocks128 >= 4 * kBigBlockRounds * 256 && a.k_blocks >= 32) ? 8 : 4;
  }
  if (a.wave_row_tiles != 8 || a.tok_tiles != 8 || dtype != SS_DTYPE_BF16 || (a.act_lo && (a.lo_row_begin % 16 || a.lo_row_end % 16)))
    a.wave_row_tiles = 4;
}

bool tile_gemm_rotates(int dtype, const TileGemmArgs &args, int head_dim) {
  TileGemmArgs a = args;
  if (a.T < 256 || a.T % 256 || a.row_tiles < 1 || a.k_blocks < 1) return false;
  choose_block(dtype, a);
  return (head_dim == 64 || head_dim == 128) && (a.wave_row_tiles * 16) % head_dim == 0;
}

ss_status launch_tile_gemm(int dtype, int epi, TileGemmArgs a, hipStream_t st) {
  if (a.T < 256 || a.T % 256) SS_FAIL(SS_EINVAL, "prefill GEMM: token count %d is not a multiple of 256", a.T);
  if (a.row_tiles < 1 || a.k_blocks < 1 || a.N < 4 || a.N % 4 || a.N > a.row_tiles * 16) SS_FAIL(SS_EINVAL, "prefill GEMM: bad shape");
  if (epi == EPI_SWIGLU && 2 * a.N != a.row_tiles * 16) SS_FAIL(SS_EINVAL, "prefill GEMM: gate/up tiles must pair up");
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
  choose_block(dtype, a);
  if (a.rope && (!a.k_cache || (a.wave_row_tiles * 16) % a.kv_Dh || (a.kv_Dh != 64 && a.kv_Dh != 128)))
    SS_FAIL(SS_EINVAL, "prefill GEMM: this block shape cannot rotate heads of %d dimensions", a.kv_Dh);
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

// ---------------------------------------------------------------------------
// Measurement aid: what the matrix cores sustain on given operand data, with and without the data movement of the
// 256-row block (one wave per SIMD, one block per compute unit, nothing else): per 64 products of 16x16x32 on halves,
// 16 LDS reads of 1 KiB back into the operand registers and 8 direct-to-LDS loads of 1 KiB.  No barrier, no epilogue.
// ---------------------------------------------------------------------------
namespace ss {
constexpr int kProbeLds = 136 * 1024;
template <bool LDSR, bool DMA>
__global__ void __launch_bounds__(256, 1) matrix_core_probe(const u32x4 *src, uint32_t src_pieces, float *out, int iters,
                                                            unsigned long long *cyc) {
  extern __shared__ __align__(16) u32x4 lds[];  // pieces 0 .. 4095: operands (read by LDSR), 4096 .. 6143: where the loads land
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  for (int i = threadIdx.x; i < 4096; i += 256) lds[i] = src[(i + blockIdx.x * 977u) % src_pieces];
  __syncthreads();
  const uint32_t base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)lds + wave * 16384 + lane * 16;
  const u32x4 *p = src + ((size_t)blockIdx.x * 4 + wave) * 512 % (src_pieces - 1024) + lane;  // 8 fragments of 64 pieces from here
  f32x4 acc[64];
  u32x4 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = lds[wave * 1024 + i * 64 + lane], b[i] = lds[wave * 1024 + (8 + i) * 64 + lane];
#pragma unroll
  for (int i = 0; i < 64; ++i) mma_f16_pinned<true>(acc[i], a[i % 8], b[i / 8]);
  const unsigned long long t0 = __builtin_readcyclecounter();
  for (int it = 0; it < iters; ++it) {
    static_for<64>([&](auto I) {
      constexpr int i = decltype(I)::value;
      mma_f16_pinned<false>(acc[i], a[i % 8], b[i / 8]);
      if constexpr (LDSR && i % 4 == 1) {  // the same values again: the registers stay what they were
        constexpr int n = i / 4;
        if constexpr (n < 8) lds_read_async<n * 1024>(a[n], base);
        else lds_read_async<n * 1024>(b[n - 8], base);
      }
      if constexpr (DMA && i % 8 == 3)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(p + (i / 8) * 64),
                                         (__attribute__((address_space(3))) void *)(lds + 4096 + (wave * 8 + i / 8) * 64), 16, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    });
    wait_lds<0>();
    if (DMA) wait_vmcnt<8>();
  }
  drain_mma();
  wait_vmcnt<0>();
  const unsigned long long t1 = __builtin_readcyclecounter();
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 64; ++i) sum += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  out[blockIdx.x * 256 + threadIdx.x] = sum;
  if (threadIdx.x == 0) cyc[blockIdx.x] = t1 - t0;
}
}  // namespace ss

extern "C" ss_status ss_debug_matrix_core_probe(const void *operands_dev, uint64_t operand_bytes, int32_t lds_reads, int32_t loads,
                                                int32_t iters, double *tflops, double *cycles_per_64, double *ghz, void *hip_stream) {
  using namespace ss;
  if (!operands_dev || operand_bytes < (1u << 20) || operand_bytes > (1ull << 32) || iters < 1 || !tflops || !cycles_per_64 || !ghz)
    SS_FAIL(SS_EINVAL, "matrix-core probe: operands of 1 MiB to 4 GiB, at least one iteration, three outputs");
  hipStream_t st = (hipStream_t)hip_stream;
  int dev = 0, cus = 0;
  SS_HIP(hipGetDevice(&dev));
  SS_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  const void *fn = lds_reads ? (loads ? (const void *)matrix_core_probe<true, true> : (const void *)matrix_core_probe<true, false>)
                             : (loads ? (const void *)matrix_core_probe<false, true> : (const void *)matrix_core_probe<false, false>);
  SS_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kProbeLds));
  float *out = nullptr;
  unsigned long long *cyc = nullptr;
  SS_HIP(hipMalloc(&out, (size_t)cus * 256 * sizeof(float)));
  if (hipMalloc(&cyc, (size_t)cus * sizeof(unsigned long long)) != hipSuccess) {
    (void)hipFree(out);
    SS_FAIL(SS_EHIP, "matrix-core probe: out of device memory");
  }
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  float ms = 0.f;
  std::vector<unsigned long long> h(cus);
  if (e == hipSuccess) e = hipEventRecord(e0, st);
  if (e == hipSuccess) {
    const u32x4 *src = (const u32x4 *)operands_dev;
    const uint32_t pieces = (uint32_t)(operand_bytes / 16);
    if (lds_reads && loads) hipLaunchKernelGGL((matrix_core_probe<true, true>), dim3(cus), dim3(256), kProbeLds, st, src, pieces, out, iters, cyc);
    else if (lds_reads) hipLaunchKernelGGL((matrix_core_probe<true, false>), dim3(cus), dim3(256), kProbeLds, st, src, pieces, out, iters, cyc);
    else if (loads) hipLaunchKernelGGL((matrix_core_probe<false, true>), dim3(cus), dim3(256), kProbeLds, st, src, pieces, out, iters, cyc);
    else hipLaunchKernelGGL((matrix_core_probe<false, false>), dim3(cus), dim3(256), kProbeLds, st, src, pieces, out, iters, cyc);
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipEventRecord(e1, st);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  if (e == hipSuccess) e = hipMemcpy(h.data(), cyc, (size_t)cus * sizeof(unsigned long long), hipMemcpyDeviceToHost);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(out);
  (void)hipFree(cyc);
  if (e != hipSuccess) SS_FAIL(SS_EHIP, "matrix-core probe: %s", hipGetErrorString(e));
  double c = 0.0;
  for (int i = 0; i < cus; ++i) c += (double)h[i];
  c /= cus;
  *tflops = 4.0 * iters * 64 * 16384.0 * cus / (ms * 1e-3) / 1e12;  // four waves a block, 64 products of 16 x 16 x 32 an iteration
  *cycles_per_64 = c / iters;
  *ghz = c / (ms * 1e-3) / 1e9;
  return SS_OK;
}

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
