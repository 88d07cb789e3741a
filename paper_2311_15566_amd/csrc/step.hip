// The whole decode step as ONE persistent kernel: 2 blocks per compute unit stay resident, walk
// the step's phase table and meet at a device-wide barrier between phases.  A phase is run by
// the same block bodies as the kernel-by-kernel path (virtual block ids instead of blockIdx), so
// both give bit-identical results.
#include <stdlib.h>

#include <algorithm>

#include "attn_block.h"
#include "rows.h"
#include "shard.h"
#include "skinny_block.h"

namespace ss {

// Barrier state in device memory (int32 words, zero at creation):
//   [0 .. 16*32)  leaf counters, one per 128-byte line     [512] root     [544] epoch     [576] abort
struct BarState {
  unsigned *leaf, *root, *epoch;
  int *abort_flag;
  int n_leaf, per_leaf;
  int spin_limit;
};

struct StepArgs {
  const Phase *phases;
  int n_phases;
  BarState bar;
};

// Counters only grow: barrier number e (counted over all launches) is complete when the root
// has reached n_leaf * e.  A block that waits longer than spin_limit polls raises the abort
// flag; every waiting block sees it and leaves, so the grid always drains.
__device__ __forceinline__ bool grid_barrier(const BarState &b, const int nblocks, const unsigned e, int *s_ok) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this thread's device-scope stores have landed
  __syncthreads();
  if (threadIdx.x == 0) {
    const int leaf = blockIdx.x / b.per_leaf;
    const unsigned members = (unsigned)min(b.per_leaf, nblocks - leaf * b.per_leaf);
    const unsigned old = __hip_atomic_fetch_add(&b.leaf[leaf * 32], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old + 1u == members * e) __hip_atomic_fetch_add(b.root, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned target = (unsigned)b.n_leaf * e;
    int it = 0, good = 1;
    while ((int)(__hip_atomic_load(b.root, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
      __builtin_amdgcn_s_sleep(1);
      if (++it > b.spin_limit || ld_dev(b.abort_flag)) {
        st_dev(b.abort_flag, 1);
        good = 0;
        break;
      }
    }
    *s_ok = good;
  }
  __syncthreads();
  return *s_ok != 0;
}

template <int NB, bool GLU, typename KT>
__global__ void __launch_bounds__(256) decode_step_persistent(StepArgs A) {
  extern __shared__ __align__(16) char smem[];
  __shared__ union {
    SkinnyShared g;
    AttnShared at;
    float scratch[4];
  } sh;
  __shared__ int s_ok;
  u32x4 *lds = (u32x4 *)smem;
  const unsigned base = *A.bar.epoch;  // barriers completed by earlier launches
  const int nblocks = gridDim.x;
  for (int p = 0; p < A.n_phases; ++p) {
    const Phase &P = A.phases[p];
    const int gx = P.gx, nvb = P.gx * P.gy, kind = P.kind;
    for (int vb = blockIdx.x; vb < nvb; vb += nblocks) {
      const int bx = vb % gx, by = vb / gx;
      if (kind == PH_EMBED) {
        __syncthreads();
        embed_row_block<bf16_t, true>(P.e, vb, sh.scratch);
      } else if (kind == PH_QKV) {
        skinny_block<bf16_t, NB, 1, PRO_NORM, EPI_F32>(P.g, bx, by, gx, lds, sh.g);
      } else if (kind == PH_ATTN) {
        decode_attn_block<KT, bf16_t, 128>(P.at, bx, by, sh.at);
      } else if (kind == PH_RESID) {
        skinny_block<bf16_t, NB, 1, PRO_ACT, EPI_RESID>(P.g, bx, by, gx, lds, sh.g);
      } else if (kind == PH_FFN_UP) {
        if (GLU) skinny_block<bf16_t, NB, 2, PRO_NORM, EPI_SWIGLU>(P.g, bx, by, gx, lds, sh.g);
        else skinny_block<bf16_t, NB, 1, PRO_NORM, EPI_ACT>(P.g, bx, by, gx, lds, sh.g);
      } else {
        skinny_block<bf16_t, NB, 1, PRO_NORM, EPI_LOGITS>(P.g, bx, by, gx, lds, sh.g);
      }
    }
    if (p + 1 < A.n_phases && !grid_barrier(A.bar, nblocks, base + (unsigned)p + 1u, &s_ok)) return;
  }
  // every block read `base` before its first arrival, and this block is past the last barrier
  if (blockIdx.x == 0 && threadIdx.x == 0) *A.bar.epoch = base + (unsigned)(A.n_phases - 1);
}

static const int kLdsBytes = 64 * 1024;

typedef void (*StepKernel)(StepArgs);
static StepKernel pick_kernel(const Shard *sh, int B) {
  const bool glu = sh->m.act == SS_ACT_SWIGLU, f16 = sh->m.kv_dtype == SS_DTYPE_F16;
  const int nb = B <= 16 ? 1 : 2;
#define SS_PICK(NB, GLU, KT) return decode_step_persistent<NB, GLU, KT>
  if (nb == 1) {
    if (glu) { if (f16) SS_PICK(1, true, f16_t); else SS_PICK(1, true, bf16_t); }
    else { if (f16) SS_PICK(1, false, f16_t); else SS_PICK(1, false, bf16_t); }
  } else {
    if (glu) { if (f16) SS_PICK(2, true, f16_t); else SS_PICK(2, true, bf16_t); }
    else { if (f16) SS_PICK(2, false, f16_t); else SS_PICK(2, false, bf16_t); }
  }
#undef SS_PICK
}

// blocks of the persistent grid, or 0 if two blocks per compute unit cannot be resident
static int persistent_grid(StepKernel k) {
  static std::map<StepKernel, int> cache;
  auto it = cache.find(k);
  if (it != cache.end()) return it->second;
  int grid = 0, occ = 0, dev = 0, cus = 0;
  if (hipGetDevice(&dev) == hipSuccess &&
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
      hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, (const void *)k, 256, kLdsBytes) == hipSuccess && occ >= 2 &&
      cus > 0)
    grid = 2 * cus;
  if (grid > 512) grid = 512;  // the barrier tree is sized for 512 blocks
  cache[k] = grid;
  return grid;
}

bool persistent_supported(const Shard *sh, int B) {
  static const bool enabled = [] {
    const char *v = getenv("SS_PERSISTENT");
    return !(v && *v == '0');
  }();
  if (!enabled || sh->m.dtype != SS_DTYPE_BF16 || sh->L.Dh != 128 || B < 1 || B > 32) return false;
  return persistent_grid(pick_kernel(sh, B)) > 0;
}

ss_status launch_persistent_step(Shard *sh, const std::vector<Phase> &plan, const GraphKey &key, hipStream_t st) {
  const Layout &L = sh->L;
  if (!plan.empty()) {
    if (plan.size() * sizeof(Phase) > L.phases_bytes) SS_FAIL(SS_EINVAL, "phase table does not fit its buffer");
    for (const Phase &ph : plan) {
      if (ph.kind == PH_ATTN) SS_TRY(check_decode_attn(ph.at));
      else if (ph.kind != PH_EMBED) {
        SS_TRY(check_skinny(sh->m.dtype, ph.g));
        if (ph.g.lds_chunk < ph.g.kb_per_split && ph.g.lds_chunk % 16) SS_FAIL(SS_EINVAL, "skinny GEMM: chunk of %d k blocks", ph.g.lds_chunk);
      }
      if (ph.gx < 1 || ph.gy < 1) SS_FAIL(SS_EINVAL, "empty phase");
    }
    sh->host_plan = plan;  // stays alive while the copy is in flight
    SS_HIP(hipMemcpyAsync(sh->ws + L.ws_phases, sh->host_plan.data(), plan.size() * sizeof(Phase),
                          hipMemcpyHostToDevice, st));
    sh->phases_key = key;
    sh->phases_valid = true;
  }
  if (!sh->phases_valid || sh->host_plan.empty()) SS_FAIL(SS_ESTATE, "no phase table");
  const int B = key.B;
  StepKernel k = pick_kernel(sh, B);
  const int grid = persistent_grid(k);
  if (grid <= 0) SS_FAIL(SS_EHIP, "persistent step: two blocks per compute unit do not fit");
  unsigned *bar = (unsigned *)(sh->ws + L.ws_bar);
  StepArgs A;
  A.phases = (const Phase *)(sh->ws + L.ws_phases);
  A.n_phases = (int)sh->host_plan.size();
  A.bar.leaf = bar, A.bar.root = bar + 512, A.bar.epoch = bar + 544, A.bar.abort_flag = (int *)(bar + 576);
  A.bar.per_leaf = 64, A.bar.n_leaf = ceil_div(grid, 64);
  A.bar.spin_limit = 1 << 16;  // ~0.1 s: the kernel must exit long before anything takes the queue for hung
  hipLaunchKernelGGL(k, dim3(grid), dim3(256), kLdsBytes, st, A);
  SS_HIP(hipGetLastError());
  return SS_OK;
}

ss_status persistent_check_abort(const Shard *sh, hipStream_t st) {
  int flag = 0;
  int *bar = (int *)(sh->ws + sh->L.ws_bar);
  SS_HIP(hipMemcpyAsync(&flag, bar + 576, 4, hipMemcpyDeviceToHost, st));
  SS_HIP(hipStreamSynchronize(st));
  if (flag) {
    // who gave up first, and how far every block's control wave had come
    std::vector<int> prog(512 + 3, 0);
    SS_HIP(hipMemcpyAsync(prog.data(), bar + 1024, 512 * 4, hipMemcpyDeviceToHost, st));
    SS_HIP(hipMemcpyAsync(prog.data() + 512, bar + 1536, 3 * 4, hipMemcpyDeviceToHost, st));
    unsigned epoch = 0;
    SS_HIP(hipMemcpyAsync(&epoch, bar + 544, 4, hipMemcpyDeviceToHost, st));
    SS_HIP(hipStreamSynchronize(st));
    int lo = prog[0], hi = prog[0], n_lo = 0, first_lo = -1;
    for (int i = 0; i < 512; ++i) lo = std::min(lo, prog[i]), hi = std::max(hi, prog[i]);
    for (int i = 0; i < 512; ++i)
      if (prog[i] == lo) {
        if (first_lo < 0) first_lo = i;
        ++n_lo;
      }
    flag = 0;
    SS_HIP(hipMemcpyAsync(bar + 576, &flag, 4, hipMemcpyHostToDevice, st));
    SS_HIP(hipStreamSynchronize(st));
    SS_FAIL(SS_EHIP,
            "a device-wide barrier of the persistent decode step timed out (block %d at barrier %d after %d polls; "
            "epoch of the launch %u; arrivals per block between %d and %d, %d blocks at the minimum, first of them %d); "
            "that step committed nothing",
            prog[512], prog[513], prog[514], epoch, lo, hi, n_lo, first_lo);
  }
  return SS_OK;
}

}  // namespace ss
