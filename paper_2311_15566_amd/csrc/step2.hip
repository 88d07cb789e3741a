// The decode step as one persistent, wave-specialised kernel (bf16 models, head_dim 128).
//
// 2 blocks of 4 waves per compute unit stay resident and walk the step's phase table.
// Waves 0-2 of a block are COMPUTE waves: they do nothing but stream 1 KiB fragments (weights,
// or K/V cache rows) into two register buffers of 16 fragments and feed the matrix cores /
// the softmax; as soon as a buffer has been consumed they refill it with the fragments of the
// block's NEXT work item, also across the device-wide barrier between phases (weights and
// committed cache rows do not depend on the step's activations), so HBM keeps streaming while
// the step's dependent chain (reduce, epilogue, barrier) runs.  Wave 3 is the CONTROL wave: it
// owns every global store, the split-K / split-sequence hand-offs, the epilogues and the
// device-wide barrier.  The compute waves never wait on anything but their own fragments,
// which keeps their in-order load counters out of the chain.
#include <limits.h>
#include <math.h>
#include <stdlib.h>

#include <algorithm>

#include "attn_block.h"
#include "mma.h"
#include "rows.h"
#include "shard.h"

namespace ss {

namespace {

constexpr int CW = 3;     // compute waves per block
constexpr int UB = 16;    // fragments per register buffer

struct BarState2 {
  unsigned *leaf, *root, *epoch;
  int *abort_flag;
  int *progress;   // [blocks]: barriers this block's control wave has arrived at (this launch)
  int *abort_rec;  // first block to give up: block, barrier, polls
  unsigned long long *trace;  // block 0's control wave: wall clock at kernel start and after each barrier
  int n_leaf, per_leaf;
  int spin_limit;
  unsigned trace_base;  // epoch at the start of the launch (host mirror)
};
struct StepArgs2 {
  const Phase *phases;
  int n_phases;
  BarState2 bar;
};

// LDS of one block: activations of the current item (dynamic) + this
template <int NB, int NWMAX>
struct Shared2 {
  f32x4 hand[CW][NB][NWMAX][64];  // GEMM accumulators of the compute waves: [wave][batch tile][weight tile][lane]
  float at_acc[CW][128];     // attention: per-wave output accumulator, running max and sum
  float at_m[CW], at_l[CW];
  float sq[128];             // attention: the (rotated) query
  float fin[8][32][2];
  int fin_i[8][32];
  int abort;
};

// the control wave's part of the device-wide barrier (one wave: no block barrier needed)
__device__ __forceinline__ bool grid_barrier_wave(const BarState2 &b, const int nblocks, const unsigned e) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the control wave's stores have landed
  int good = 1;
  if ((threadIdx.x & 63) == 0) {
    const int leaf = blockIdx.x / b.per_leaf;
    const unsigned members = (unsigned)min(b.per_leaf, nblocks - leaf * b.per_leaf);
    st_dev(&b.progress[blockIdx.x], (int)e);
    const unsigned old = __hip_atomic_fetch_add(&b.leaf[leaf * 32], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old + 1u == members * e) __hip_atomic_fetch_add(b.root, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned target = (unsigned)b.n_leaf * e;
    int it = 0;
    while ((int)(__hip_atomic_load(b.root, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
      __builtin_amdgcn_s_sleep(1);
      if (++it > b.spin_limit || ld_dev(b.abort_flag)) {
        if (__hip_atomic_exchange(b.abort_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) {
          st_dev(&b.abort_rec[0], (int)blockIdx.x);
          st_dev(&b.abort_rec[1], (int)e);
          st_dev(&b.abort_rec[2], it);
        }
        good = 0;
        break;
      }
    }
  }
  if (blockIdx.x == 0 && (threadIdx.x & 63) == 0 && b.trace) b.trace[e - (unsigned)b.trace[63]] = wall_clock64();
  return __shfl(good, 0) != 0;
}

// last-arriver test for one wave (the block version is arrive_last)
__device__ __forceinline__ bool arrive_last_wave(int *counter, int expected) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  int last = 0;
  if ((threadIdx.x & 63) == 0) {
    const int old = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    last = old == expected - 1;
    if (last) st_dev(counter, 0);
  }
  return __shfl(last, 0) != 0;
}

// ---------------------------------------------------------------------------
// work items
// ---------------------------------------------------------------------------
struct Item {
  int p;   // phase index, or n_phases when there is none
  int vb;  // virtual block within the phase
  int c;   // GEMM: chunk of the block's K range (a block walks its chunks in order, accumulating)
};

// chunks of virtual block vb of a GEMM phase
__device__ __forceinline__ int item_chunks(const Phase &P, int vb) {
  if (P.kind == PH_ATTN || P.kind == PH_EMBED) return 1;
  const int by = vb / P.gx;
  const int nks = min(P.g.kb_per_split, P.g.k_blocks - by * P.g.kb_per_split);
  return (nks + P.g.lds_chunk - 1) / P.g.lds_chunk;
}

__device__ __forceinline__ Item next_item(const StepArgs2 &A, Item it, const int nblocks) {
  // the block's items: for each phase in order, vb = blockIdx.x, blockIdx.x + nblocks, ...; for
  // each vb its chunks in order
  if (it.p < A.n_phases && it.vb >= 0 && it.c + 1 < item_chunks(A.phases[it.p], it.vb)) return Item{it.p, it.vb, it.c + 1};
  int p = it.p, vb = it.vb + nblocks;
  while (p < A.n_phases) {
    if (A.phases[p].kind != PH_EMBED && vb < A.phases[p].gx * A.phases[p].gy) return Item{p, vb, 0};
    ++p;
    vb = blockIdx.x;
  }
  return Item{A.n_phases, 0, 0};
}

// What one compute wave streams for an item: nf fragments; fragment f lives at base + f_off(f).
struct Stream {
  const u32x4 *base;   // lane-adjusted
  int nf;              // fragments of this wave
  int kind;            // PH_*
  int nw;              // GEMM: weight tiles per wave
  int k_blocks;        // GEMM: fragment stride between the weight tiles of a pair
  int rg_stride;       // ATTN: fragments between two of this wave's row groups
  const u32x4 *vbase;  // ATTN: V rows (K rows at base)
  int last_row_off;    // ATTN: fragment offset clamp (rows beyond the committed length are not read)
};

template <bool GLU>
__device__ __forceinline__ Stream make_stream(const StepArgs2 &A, const Item it, const int wave, const int lane) {
  Stream s;
  s.nf = 0, s.base = nullptr, s.vbase = nullptr, s.kind = -1, s.nw = 1, s.k_blocks = 0, s.rg_stride = 0, s.last_row_off = 0;
  if (it.p >= A.n_phases || wave >= CW) return s;
  const Phase &P = A.phases[it.p];
  s.kind = P.kind;
  const int bx = it.vb % P.gx, by = it.vb / P.gx;
  if (P.kind == PH_ATTN) {
    const DecodeAttnArgs &a = P.at;
    const int b = bx / a.Hs, h = bx - b * a.Hs;
    const int n = a.lens[b];
    const int r0 = by * a.rows_per_block, r1 = min(r0 + a.rows_per_block, n);
    if (r1 <= r0) return s;
    const int groups = (r1 - r0 + 3) >> 2;                       // row groups of 4 rows = 1 KiB
    const int mine = wave < groups ? (groups - wave + CW - 1) / CW : 0;
    s.nf = 2 * mine;
    const size_t off = (size_t)b * a.row_stride + (size_t)h * a.head_stride + (size_t)r0 * 256;
    s.base = (const u32x4 *)(a.k_cache + off) + wave * 64 + lane;
    s.vbase = (const u32x4 *)(a.v_cache + off) + wave * 64 + lane;
    s.rg_stride = CW * 64;
    // lane's row within a group = lane / 16; rows >= r1 are clamped onto row r1 - 1
    s.last_row_off = (r1 - 1 - r0) * 16 + (lane & 15) - (wave * 64 + lane);
    return s;
  }
  const SkinnyArgs &a = P.g;
  const int task = bx * CW + wave;
  if (task >= a.tasks) return s;
  const int nks = min(a.kb_per_split, a.k_blocks - by * a.kb_per_split);
  const int kb0 = by * a.kb_per_split + it.c * a.lds_chunk;
  const int nk = min(a.lds_chunk, nks - it.c * a.lds_chunk);
  s.nw = (GLU && P.kind == PH_FFN_UP) ? 2 : 1;
  s.k_blocks = a.k_blocks;
  s.nf = nk * s.nw;
  s.base = (const u32x4 *)a.w + ((size_t)task * s.nw * a.k_blocks + kb0) * 64 + lane;
  return s;
}

// issue the loads of fragments [f0, f0 + UB) of a stream into a register buffer
__device__ __forceinline__ void load_buf(u32x4 (&buf)[UB], const Stream &s, const int f0) {
#pragma unroll
  for (int u = 0; u < UB; ++u) {
    const int f = f0 + u;
    if (f < s.nf) {
      if (s.kind == PH_ATTN) {
        const int rg = f >> 1;
        int off = rg * s.rg_stride;
        off = min(off, s.last_row_off);
        buf[u] = __builtin_nontemporal_load(((f & 1) ? s.vbase : s.base) + off);
      } else {
        const int j = s.nw == 2 ? (f & 1) : 0, kb = s.nw == 2 ? (f >> 1) : f;
        buf[u] = __builtin_nontemporal_load(s.base + ((size_t)j * s.k_blocks + kb) * 64);
      }
    } else {
      buf[u] = u32x4{0u, 0u, 0u, 0u};
    }
  }
}

template <typename KT>
__device__ __forceinline__ void unpack_kv(const u32x4 &raw, float *out) { unpack16<KT>(raw, out); }

}  // namespace

// ---------------------------------------------------------------------------
// the kernel
// ---------------------------------------------------------------------------
template <int NB, bool GLU, typename KT>
__global__ void __launch_bounds__(256, 2) decode_step_persistent2(StepArgs2 A) {
  typedef bf16_t T;
  constexpr int PL = 8, FK = 32, AP = 2;
  extern __shared__ __align__(16) char smem[];
  constexpr int NWMAX = GLU ? 2 : 1;
  __shared__ Shared2<NB, NWMAX> sh;
  u32x4 *lds = (u32x4 *)smem;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool control = wave == CW;
  const int nblocks = gridDim.x;
  const unsigned base_epoch = *A.bar.epoch;
  if (tid == 0) sh.abort = 0;
  if (blockIdx.x == 0 && tid == 0 && A.bar.trace) A.bar.trace[0] = wall_clock64(), A.bar.trace[63] = base_epoch;

  // ---- phase 0: the embedding, by the control waves of the first B blocks ----
  Item it = next_item(A, Item{0, (int)blockIdx.x - nblocks, 0}, nblocks);  // first non-embedding item
  Stream st = make_stream<GLU>(A, it, wave, lane);
  u32x4 bufA[UB], bufB[UB];
  if (!control) {
    load_buf(bufA, st, 0);
    load_buf(bufB, st, UB);
  } else {
    const Phase &P0 = A.phases[0];
    if (P0.kind == PH_EMBED) {
      for (int r = blockIdx.x; r < P0.gx; r += nblocks) {
        // one wave: 16-byte pieces strided over the row, two-pass statistics from registers
        const EmbedArgs &e = P0.e;
        int tok = e.tokens[r];
        tok = min(max(tok, 0), e.V - 1);
        const int pos = e.lens ? e.lens[r] : (r % e.S);
        const int nvec = e.d / PL;
        const u32x4 *te = (const u32x4 *)((const T *)e.wte + (size_t)tok * e.d);
        const u32x4 *pe = e.wpe ? (const u32x4 *)((const T *)e.wpe + (size_t)pos * e.d) : nullptr;
        float s1 = 0.f;
        for (int v = lane; v < nvec; v += 64) {
          float x[PL];
          widen16<T>(te[v], x);
          if (pe) {
            float q[PL];
            widen16<T>(pe[v], q);
#pragma unroll
            for (int k = 0; k < PL; ++k) x[k] += q[k];
          }
          float *xo = e.x + (size_t)r * e.d + (size_t)v * PL;
#pragma unroll
          for (int k = 0; k < PL; ++k) s1 += x[k], st_dev(xo + k, x[k]);
        }
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) s1 += __shfl_xor(s1, off);
        const float mean = e.rms ? 0.f : s1 / (float)e.d;
        float s2 = 0.f;
        for (int v = lane; v < nvec; v += 64) {  // second pass re-reads the table rows (cached)
          float x[PL];
          widen16<T>(te[v], x);
          if (pe) {
            float q[PL];
            widen16<T>(pe[v], q);
#pragma unroll
            for (int k = 0; k < PL; ++k) x[k] += q[k];
          }
#pragma unroll
          for (int k = 0; k < PL; ++k) s2 += (x[k] - mean) * (x[k] - mean);
        }
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) s2 += __shfl_xor(s2, off);
        if (lane == 0) {
          st_dev(&e.stats[r * 2], mean);
          st_dev(&e.stats[r * 2 + 1], rsqrtf(s2 / (float)e.d + e.eps));
        }
      }
    }
  }

  int cur_phase = 0;  // the phase whose leading barrier the control wave has passed
  f32x4 acc[NB][2];   // GEMM accumulators of a compute wave, carried over the chunks of an item
  while (it.p < A.n_phases) {
    const Phase &P = A.phases[it.p];
    const int kind = P.kind;
    const int bx = it.vb % P.gx, by = it.vb / P.gx;

    // ---- B0: the control wave brings the block up to this item's phase ----
    if (control) {
      int ok = 1;
      while (ok && cur_phase < it.p) {
        ok = grid_barrier_wave(A.bar, nblocks, base_epoch + (unsigned)cur_phase + 1u);
        ++cur_phase;
      }
      if (!ok && lane == 0) sh.abort = 1;
    }
    __syncthreads();
    if (sh.abort) return;

    if (kind == PH_ATTN) {
      // =====================================================================
      // decode attention: (b, h) = bx, rows [r0, r1) of the committed cache
      // =====================================================================
      const DecodeAttnArgs &a = P.at;
      const int b = bx / a.Hs, h = bx - b * a.Hs;
      const int n = a.lens[b];
      const int live_splits = max(1, (n + a.rows_per_block - 1) / a.rows_per_block);
      const int HD = a.Hs * 128;
      const float scale = rsqrtf(128.f);
      const float2 *tab = a.rope ? a.rope + (size_t)n * 64 : nullptr;
      const float *qraw = a.qkv + (size_t)b * 3 * HD + h * 128;
      const bool live_item = by < live_splits;
      if (live_item && control) {  // the query, rotated, into LDS
        sh.sq[lane] = rope_elem(qraw, lane, 64, tab);
        sh.sq[lane + 64] = rope_elem(qraw, lane + 64, 64, tab);
      }
      __syncthreads();  // B1
      if (live_item && !control) {
        const int r0 = by * a.rows_per_block, r1 = min(r0 + a.rows_per_block, n);
        const int c = lane & 15, g = lane >> 4;
        float qf[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[e] = sh.sq[c * 8 + e];
        float m = -1e30f, l = 0.f, acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
        auto consume = [&](u32x4(&buf)[UB], int f0) {
          // UB fragments = UB/2 row groups (K, V pairs); lane group g owns row 4*rg + g of each
          float s[UB / 2];
          float mb = -1e30f;
#pragma unroll
          for (int u = 0; u < UB / 2; ++u) {
            const int f = f0 + 2 * u;
            const int rg = wave + CW * (f >> 1);
            const int row = r0 + 4 * rg + g;
            float kf[8];
            unpack_kv<KT>(buf[2 * u], kf);
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) d += qf[e] * kf[e];
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) d += __shfl_xor(d, off);
            s[u] = (f < st.nf && row < r1) ? d * scale : -INFINITY;
            mb = fmaxf(mb, s[u]);
          }
          const float mn = fmaxf(m, mb);
          const float alpha = __expf(m - mn);
          l *= alpha;
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[e] *= alpha;
#pragma unroll
          for (int u = 0; u < UB / 2; ++u) {
            const float p = __expf(s[u] - mn);
            l += p;
            float vf[8];
            unpack_kv<KT>(buf[2 * u + 1], vf);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += p * vf[e];
          }
          m = mn;
        };
        const Item nit = next_item(A, it, nblocks);
        const Stream nst = make_stream<GLU>(A, nit, wave, lane);
        if (st.nf > 0) consume(bufA, 0);
        load_buf(bufA, nst, 0);
        if (st.nf > UB) consume(bufB, UB);
        load_buf(bufB, nst, UB);
        // merge the 4 lane groups of the wave
#pragma unroll
        for (int off = 16; off < 64; off <<= 1) {
          const float mo = __shfl_xor(m, off), lo = __shfl_xor(l, off);
          const float mn = fmaxf(m, mo);
          const float f0 = __expf(m - mn), f1 = __expf(mo - mn);
          l = l * f0 + lo * f1;
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[e] = acc[e] * f0 + __shfl_xor(acc[e], off) * f1;
          m = mn;
        }
        if (lane < 16) {
#pragma unroll
          for (int e = 0; e < 8; ++e) sh.at_acc[wave][lane * 8 + e] = acc[e];
          if (lane == 0) sh.at_m[wave] = m, sh.at_l[wave] = l;
        }
        st = nst;
        it = nit;
      } else if (!control) {  // an item past the live splits: nothing to stream
        const Item nit = next_item(A, it, nblocks);
        const Stream nst = make_stream<GLU>(A, nit, wave, lane);
        load_buf(bufA, nst, 0);
        load_buf(bufB, nst, UB);
        st = nst;
        it = nit;
      }
      __syncthreads();  // B2
      if (control) {
        if (live_item) {
          // thread pair (lane, lane + 64) -> output dims lane and lane + 64
          float M[2], Ls[2], Aq[2];
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            const int e = lane + 64 * q;
            M[q] = -1e30f, Ls[q] = 0.f, Aq[q] = 0.f;
#pragma unroll
            for (int w = 0; w < CW; ++w) M[q] = fmaxf(M[q], sh.at_m[w]);
#pragma unroll
            for (int w = 0; w < CW; ++w) {
              const float f = __expf(sh.at_m[w] - M[q]);
              Ls[q] += sh.at_l[w] * f;
              Aq[q] += sh.at_acc[w][e] * f;
            }
          }
          float *part = a.part + ((size_t)bx * a.splits) * 132;
          bool last = true;
          if (live_splits > 1) {
            float *p = part + (size_t)by * 132;
            st_dev(p + lane, Aq[0]);
            st_dev(p + lane + 64, Aq[1]);
            if (lane == 0) st_dev(p + 128, M[0]), st_dev(p + 129, Ls[0]);
            last = arrive_last_wave(&a.counters[bx], live_splits);
            if (last) {
#pragma unroll
              for (int q = 0; q < 2; ++q) M[q] = -1e30f, Ls[q] = 0.f, Aq[q] = 0.f;
              for (int s2 = 0; s2 < live_splits; ++s2) M[0] = fmaxf(M[0], ld_dev(part + (size_t)s2 * 132 + 128));
              M[1] = M[0];
              for (int s2 = 0; s2 < live_splits; ++s2) {
                const float *p2 = part + (size_t)s2 * 132;
                const float f = __expf(ld_dev(p2 + 128) - M[0]);
                const float ll = ld_dev(p2 + 129) * f;
                Ls[0] += ll, Ls[1] += ll;
                Aq[0] += ld_dev(p2 + lane) * f;
                Aq[1] += ld_dev(p2 + lane + 64) * f;
              }
            }
          }
          if (last) {
            // the new token: append as row n (committed by the step's last phase), attend to itself
            float prod = 0.f, vnew[2];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
              const int e = lane + 64 * q;
              const float kn = rope_elem(qraw + HD, e, 64, tab);
              const KT kt = Elem<KT>::from_f32(kn);
              const KT vt = Elem<KT>::from_f32(qraw[2 * HD + e]);
              const size_t off = (size_t)b * a.row_stride + (size_t)h * a.head_stride + (size_t)n * 256;
              ((KT *)(a.k_cache + off))[e] = kt;
              ((KT *)(a.v_cache + off))[e] = vt;
              vnew[q] = Elem<KT>::to_f32(vt);
              prod += sh.sq[e] * Elem<KT>::to_f32(kt);
            }
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) prod += __shfl_xor(prod, off);
            const float sn = prod * scale;
            float o[2];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
              const float mn = fmaxf(M[q], sn);
              const float f0 = __expf(M[q] - mn), p = __expf(sn - mn);
              o[q] = (Aq[q] * f0 + p * vnew[q]) / (Ls[q] * f0 + p);
            }
            // operand buffer in whole words: even lanes pack dims (e, e + 1)
#pragma unroll
            for (int q = 0; q < 2; ++q) {
              const float o_next = __shfl_xor(o[q], 1);
              if ((lane & 1) == 0) {
                const int k = h * 128 + lane + 64 * q;
                const T h0 = Elem<T>::from_f32(o[q]), h1 = Elem<T>::from_f32(o_next);
#pragma unroll
                for (int part_i = 0; part_i < AP; ++part_i) {
                  T w2[2];
                  w2[0] = part_i == 0 ? h0 : Elem<T>::from_f32(o[q] - Elem<T>::to_f32(h0));
                  w2[1] = part_i == 0 ? h1 : Elem<T>::from_f32(o_next - Elem<T>::to_f32(h1));
                  uint32_t word;
                  __builtin_memcpy(&word, w2, 4);
                  st_dev((uint32_t *)((T *)a.o_out + frag_offset_parts<T>(b, k, HD / FK, AP, part_i)), word);
                }
              }
            }
          }
        }
        it = next_item(A, it, nblocks);
      }
      continue;
    }

    // =======================================================================
    // skinny GEMM item: tasks bx*3 .. bx*3+2, K range by
    // =======================================================================
    const SkinnyArgs &a = P.g;
    const int nks = min(a.kb_per_split, a.k_blocks - by * a.kb_per_split);
    const int kb0 = by * a.kb_per_split + it.c * a.lds_chunk;
    const int nk = min(a.lds_chunk, nks - it.c * a.lds_chunk);
    const bool first_chunk = it.c == 0, last_chunk = (it.c + 1) * a.lds_chunk >= nks;
    const int K = a.k_blocks * FK;
    const bool glu = GLU && kind == PH_FFN_UP;
    // ---- stage the activations of the K range (all four waves) ----
    if (kind == PH_RESID) {
      const u32x4 *src = (const u32x4 *)a.act;
      const int per = nk * AP * 64;
      for (int i = tid; i < NB * per; i += 256) {
        const int t = i / per, r = i - t * per;
        if (t * 16 + (r & 15) < a.B) lds[t * a.lds_chunk * AP * 64 + r] = src[((size_t)t * a.k_blocks + kb0) * AP * 64 + r];
      }
    } else {
      const int ppr = nk * 4;
      for (int i = tid; i < a.B * ppr; i += 256) {
        const int row = i / ppr, p = i - row * ppr;
        const int k0 = kb0 * FK + p * PL;
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
            v[1][q * 4 + e] = Elem<T>::from_f32(y[e] - Elem<T>::to_f32(v[0][q * 4 + e]));
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
    __syncthreads();  // B1
    if (!control) {
      if (first_chunk) {
#pragma unroll
        for (int t = 0; t < NB; ++t) acc[t][0] = acc[t][1] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
      auto consume = [&](u32x4(&buf)[UB], int f0) {
#pragma unroll
        for (int u = 0; u < UB; ++u) {
          const int f = f0 + u;
          if (f < st.nf) {
            const int kb = glu ? (f >> 1) : f;
#pragma unroll
            for (int t = 0; t < NB; ++t)
#pragma unroll
              for (int part = 0; part < AP; ++part) {
                const u32x4 af = lds[((t * a.lds_chunk + kb) * AP + part) * 64 + lane];
                if (glu && (u & 1)) acc[t][1] = Mma<T>::mma(buf[u], af, acc[t][1]);
                else acc[t][0] = Mma<T>::mma(buf[u], af, acc[t][0]);
              }
          }
        }
      };
      const Item nit = next_item(A, it, nblocks);
      const Stream nst = make_stream<GLU>(A, nit, wave, lane);
      consume(bufA, 0);
      load_buf(bufA, nst, 0);
      consume(bufB, UB);
      load_buf(bufB, nst, UB);
      if (last_chunk) {
#pragma unroll
        for (int t = 0; t < NB; ++t) {
          sh.hand[wave][t][0][lane] = acc[t][0];
          if (GLU) sh.hand[wave][t][NWMAX - 1][lane] = acc[t][1];
        }
      }
      st = nst;
      it = nit;
    }
    __syncthreads();  // B2
    if (control && !last_chunk) it = next_item(A, it, nblocks);
    if (control && last_chunk) {
      const int ngroups = P.gx;
      const int q4 = (lane >> 4) * 4, bl = lane & 15;
      const int NWr = glu ? 2 : 1;
      const size_t npad = (size_t)a.tasks * NWr * 16;
      bool last = true;
      if (a.split > 1) {
#pragma unroll 1
        for (int w = 0; w < CW; ++w) {
          const int task = bx * CW + w;
          if (task < a.tasks) {
#pragma unroll
            for (int t = 0; t < NB; ++t)
              if (t * 16 + bl < a.B) {
#pragma unroll
                for (int j = 0; j < NWMAX; ++j)
                  if (j < NWr) {
                    const f32x4 v = sh.hand[w][t][j][lane];
                    float *p = a.splitk + ((size_t)by * NB * 16 + t * 16 + bl) * npad + (size_t)(task * NWr + j) * 16 + q4;
#pragma unroll
                    for (int i = 0; i < 4; ++i) st_dev(p + i, v[i]);
                  }
              }
          }
        }
        last = arrive_last_wave(&a.counters[bx], a.split);
      }
      if (last) {
        float s1[NB], s2[NB], bv[NB];
        int bi[NB];
#pragma unroll
        for (int t = 0; t < NB; ++t) s1[t] = 0.f, s2[t] = 0.f, bv[t] = -INFINITY, bi[t] = INT_MAX;
#pragma unroll 1
        for (int w = 0; w < CW; ++w) {
          const int task = bx * CW + w, n0 = task * 16 + q4;
          if (task >= a.tasks) continue;
          // this tile's sums: straight from the compute wave, or the partials in split order
          f32x4 acc[NB][NWMAX];
#pragma unroll
          for (int t = 0; t < NB; ++t)
#pragma unroll
            for (int j = 0; j < NWMAX; ++j) {
              acc[t][j] = f32x4{0.f, 0.f, 0.f, 0.f};
              if (j >= NWr || t * 16 + bl >= a.B) continue;
              if (a.split == 1) {
                acc[t][j] = sh.hand[w][t][j][lane];
              } else {
                f32x4 sum = f32x4{0.f, 0.f, 0.f, 0.f};
                const float *p0 = a.splitk + ((size_t)t * 16 + bl) * npad + (size_t)(task * NWr + j) * 16 + q4;
                const size_t sstride = (size_t)NB * 16 * npad;
                int s3 = 0;
                for (; s3 + 4 <= a.split; s3 += 4) {
                  float v[4][4];
#pragma unroll
                  for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[r][i] = ld_dev(p0 + (size_t)(s3 + r) * sstride + i);
#pragma unroll
                  for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int i = 0; i < 4; ++i) sum[i] += v[r][i];
                }
                for (; s3 < a.split; ++s3)
#pragma unroll
                  for (int i = 0; i < 4; ++i) sum[i] += ld_dev(p0 + (size_t)s3 * sstride + i);
                acc[t][j] = sum;
              }
            }
#pragma unroll
          for (int t = 0; t < NB; ++t) {
            const int b = t * 16 + bl;
            if (kind == PH_QKV) {
              if (b < a.B) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                  const int n = n0 + i;
                  if (n < a.N) st_dev(&a.out_f32[(size_t)b * a.ld_out + n], acc[t][0][i] + (a.bias ? a.bias[n] : 0.f));
                }
              }
            } else if (kind == PH_FFN_UP) {
              if (b < a.B && n0 < a.N) {
                float u[4];
#pragma unroll
                for (int i = 0; i < 4; ++i)
                  u[i] = glu ? silu_f(acc[t][0][i]) * acc[t][NWMAX - 1][i]
                             : act_apply(a.act_kind, acc[t][0][i] + (a.bias ? a.bias[n0 + i] : 0.f));
                store4_frag<T, true>(a.act_out, b, n0, a.out_k_blocks, AP, u);
              }
            } else if (kind == PH_RESID) {
              if (b < a.B) {
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
            } else {  // PH_LM_HEAD
#pragma unroll
              for (int i = 0; i < 4; ++i) {
                const int n = n0 + i;
                if (n < a.N) {
                  const float v = acc[t][0][i];
                  if (a.out_f32 && b < a.B) a.out_f32[(size_t)b * a.ld_out + n] = v;
                  if (v > bv[t]) bv[t] = v, bi[t] = n;
                }
              }
            }
          }
        }
        if (kind == PH_RESID) {
#pragma unroll
          for (int t = 0; t < NB; ++t) {
            s1[t] += __shfl_xor(s1[t], 16);
            s2[t] += __shfl_xor(s2[t], 16);
            s1[t] += __shfl_xor(s1[t], 32);
            s2[t] += __shfl_xor(s2[t], 32);
            if (lane < 16) {
              st_dev(&a.stat_part[((size_t)bx * 32 + t * 16 + lane) * 2 + 0], s1[t]);
              st_dev(&a.stat_part[((size_t)bx * 32 + t * 16 + lane) * 2 + 1], s2[t]);
            }
          }
          if (arrive_last_wave(&a.counters[ngroups], ngroups)) {
            // lane (b = lane % 32, half = lane / 32) sums the groups of its half in 4 interleaved
            // slices; the 8 slices are then added in slice order
            const int b = lane & 31, half = lane >> 5;
            float t1[4] = {0.f, 0.f, 0.f, 0.f}, t2[4] = {0.f, 0.f, 0.f, 0.f};
            if (b < a.B) {
              for (int g0 = half * 4; g0 < ngroups; g0 += 8) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                  if (g0 + q < ngroups) {
                    t1[q] += ld_dev(&a.stat_part[((size_t)(g0 + q) * 32 + b) * 2 + 0]);
                    t2[q] += ld_dev(&a.stat_part[((size_t)(g0 + q) * 32 + b) * 2 + 1]);
                  }
                }
              }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) sh.fin[half * 4 + q][b][0] = t1[q], sh.fin[half * 4 + q][b][1] = t2[q];
            __builtin_amdgcn_wave_barrier();  // LDS operations of one wave execute in order
            if (lane < a.B) {
              float u1 = 0.f, u2 = 0.f;
#pragma unroll
              for (int q = 0; q < 8; ++q) u1 += sh.fin[q][lane][0], u2 += sh.fin[q][lane][1];
              const float inv = 1.0f / (float)a.N;
              float mean = u1 * inv;
              const float ms = u2 * inv;
              float rstd;
              if (a.rms) {
                rstd = rsqrtf(ms + a.eps);
                mean = 0.f;
              } else {
                rstd = rsqrtf(fmaxf(ms - mean * mean, 0.f) + a.eps);
              }
              st_dev(&a.stats_out[lane * 2 + 0], mean);
              st_dev(&a.stats_out[lane * 2 + 1], rstd);
            }
          }
        } else if (kind == PH_LM_HEAD) {
#pragma unroll
          for (int t = 0; t < NB; ++t) {
#pragma unroll
            for (int off = 16; off <= 32; off <<= 1) {
              const float ov = __shfl_xor(bv[t], off);
              const int oi = __shfl_xor(bi[t], off);
              if (ov > bv[t] || (ov == bv[t] && oi < bi[t])) bv[t] = ov, bi[t] = oi;
            }
            if (lane < 16) {
              st_dev(&a.am_val[(size_t)bx * 32 + t * 16 + lane], bv[t]);
              st_dev(&a.am_idx[(size_t)bx * 32 + t * 16 + lane], bi[t]);
            }
          }
          if (arrive_last_wave(&a.counters[ngroups], ngroups)) {
            const int b = lane & 31, half = lane >> 5;
            float fv = -INFINITY;
            int fi = INT_MAX;
            if (b < a.B) {
#pragma unroll 4
              for (int g = half; g < ngroups; g += 2) {
                const float ov = ld_dev(&a.am_val[(size_t)g * 32 + b]);
                const int oi = ld_dev(&a.am_idx[(size_t)g * 32 + b]);
                if (ov > fv || (ov == fv && oi < fi)) fv = ov, fi = oi;
              }
            }
            const float ov = __shfl_xor(fv, 32);
            const int oi = __shfl_xor(fi, 32);
            if (ov > fv || (ov == fv && oi < fi)) fv = ov, fi = oi;
            if (lane < a.B) {
              if (a.next_tokens) a.next_tokens[lane] = fi;
              // token-level commit: the last action of the step
              for (int q = 0; q < a.n_lens; ++q) a.lens[q][lane] += a.commit_inc;
            }
          }
        }
      }
      it = next_item(A, it, nblocks);
    }
  }

  // the control wave still owes the barriers of the phases in which this block had no item
  if (control) {
    int ok = 1;
    while (ok && cur_phase < A.n_phases - 1) {
      ok = grid_barrier_wave(A.bar, nblocks, base_epoch + (unsigned)cur_phase + 1u);
      ++cur_phase;
    }
    if (blockIdx.x == 0 && lane == 0 && ok) {
      *A.bar.epoch = base_epoch + (unsigned)(A.n_phases - 1);
      if (A.bar.trace) A.bar.trace[A.n_phases] = wall_clock64();
    }
  }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
static int lds_bytes2(int B) { return (B <= 16 ? 64 : 56) * 1024; }  // + static LDS <= 80 KiB: two blocks per CU
typedef void (*StepKernel2)(StepArgs2);

static StepKernel2 pick_kernel2(const Shard *sh, int B) {
  const bool glu = sh->m.act == SS_ACT_SWIGLU, f16 = sh->m.kv_dtype == SS_DTYPE_F16;
  const int nb = B <= 16 ? 1 : 2;
#define SS_PICK(NB, GLU, KT) return decode_step_persistent2<NB, GLU, KT>
  if (nb == 1) {
    if (glu) { if (f16) SS_PICK(1, true, f16_t); else SS_PICK(1, true, bf16_t); }
    else { if (f16) SS_PICK(1, false, f16_t); else SS_PICK(1, false, bf16_t); }
  } else {
    if (glu) { if (f16) SS_PICK(2, true, f16_t); else SS_PICK(2, true, bf16_t); }
    else { if (f16) SS_PICK(2, false, f16_t); else SS_PICK(2, false, bf16_t); }
  }
#undef SS_PICK
}

static int persistent_grid2(StepKernel2 k, int B) {
  static std::map<StepKernel2, int> cache;
  auto it = cache.find(k);
  if (it != cache.end()) return it->second;
  int grid = 0, occ = 0, dev = 0, cus = 0;
  if (hipGetDevice(&dev) == hipSuccess &&
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
      hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, (const void *)k, 256, lds_bytes2(B)) == hipSuccess && occ >= 2 &&
      cus > 0)
    grid = std::min(2 * cus, 512);  // the barrier tree is sized for 512 blocks
  if (grid > 0) {
    const char *v = getenv("SS_PERSISTENT_BLOCKS");  // fewer resident blocks (testing aid)
    if (v && atoi(v) > 0) grid = std::min(grid, atoi(v));
  }
  cache[k] = grid;
  return grid;
}

int persistent2_blocks(const Shard *sh, int B) {
  if (sh->m.dtype != SS_DTYPE_BF16 || sh->L.Dh != 128 || B < 1 || B > 32) return 0;
  return persistent_grid2(pick_kernel2(sh, B), B);
}

ss_status launch_persistent2_step(Shard *sh, const std::vector<Phase> &plan, const GraphKey &key, hipStream_t stream) {
  const Layout &L = sh->L;
  if (!plan.empty()) {
    if (plan.size() * sizeof(Phase) > L.phases_bytes) SS_FAIL(SS_EINVAL, "phase table does not fit its buffer");
    for (const Phase &ph : plan) {
      if (ph.gx < 1 || ph.gy < 1) SS_FAIL(SS_EINVAL, "empty phase");
      if (ph.kind == PH_ATTN) {
        SS_TRY(check_decode_attn(ph.at));
        if (ph.at.rows_per_block > 4 * 2 * (UB / 2) * CW || ph.at.Dh != 128)
          SS_FAIL(SS_EINVAL, "persistent step: %d rows per attention block exceed what three waves hold", ph.at.rows_per_block);
      } else if (ph.kind != PH_EMBED) {
        SS_TRY(check_skinny(sh->m.dtype, ph.g));
        const int nw = (ph.kind == PH_FFN_UP && sh->m.act == SS_ACT_SWIGLU) ? 2 : 1;
        if (ph.g.lds_chunk * nw > 2 * UB)
          SS_FAIL(SS_EINVAL, "persistent step: %d fragments per wave and chunk exceed the register buffers", ph.g.lds_chunk * nw);
        if ((size_t)ph.g.nb * ph.g.lds_chunk * 2 * 1024 > (size_t)lds_bytes2(key.B))
          SS_FAIL(SS_EINVAL, "persistent step: a chunk of %d k blocks does not fit the LDS", ph.g.lds_chunk);
        if (ph.gx != ceil_div(ph.g.tasks, CW) || ph.gy != ph.g.split) SS_FAIL(SS_EINVAL, "persistent step: bad grid");
      }
    }
    if (plan[0].kind != PH_EMBED || plan.size() < 2) SS_FAIL(SS_EINVAL, "persistent step: plan must start with the embedding");
    sh->host_plan = plan;
    SS_HIP(hipMemcpyAsync(sh->ws + L.ws_phases, sh->host_plan.data(), plan.size() * sizeof(Phase),
                          hipMemcpyHostToDevice, stream));
    sh->phases_key = key;
    sh->phases_valid = true;
  }
  if (!sh->phases_valid || sh->host_plan.empty()) SS_FAIL(SS_ESTATE, "no phase table");
  StepKernel2 k = pick_kernel2(sh, key.B);
  const int grid = persistent_grid2(k, key.B);
  if (grid <= 0) SS_FAIL(SS_EHIP, "persistent step: two blocks per compute unit do not fit");
  unsigned *bar = (unsigned *)(sh->ws + L.ws_bar);
  StepArgs2 A;
  A.phases = (const Phase *)(sh->ws + L.ws_phases);
  A.n_phases = (int)sh->host_plan.size();
  A.bar.leaf = bar, A.bar.root = bar + 512, A.bar.epoch = bar + 544, A.bar.abort_flag = (int *)(bar + 576);
  A.bar.progress = (int *)(bar + 1024), A.bar.abort_rec = (int *)(bar + 1536);
  A.bar.trace = getenv("SS_TRACE") ? (unsigned long long *)(sh->ws + L.ws_trace) : nullptr;
  A.bar.trace_base = 0;
  A.bar.per_leaf = 64, A.bar.n_leaf = ceil_div(grid, 64);
  // a poll takes about a microsecond: a barrier that has not completed after ~0.1 s never will,
  // and the kernel must be gone long before anything takes the queue for hung
  A.bar.spin_limit = 1 << 16;
  hipLaunchKernelGGL(k, dim3(grid), dim3(256), lds_bytes2(key.B), stream, A);
  SS_HIP(hipGetLastError());
  return SS_OK;
}

}  // namespace ss
