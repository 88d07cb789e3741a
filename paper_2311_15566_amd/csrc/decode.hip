// The decode step and the initial phase: row kernels (embedding, norms) and the launch
// sequence over a group of co-resident shards, with HIP-graph replay of the decode step.
#include <stdlib.h>
#include <string.h>

#include <math.h>

#include <algorithm>
#include <atomic>
#include <mutex>
#include <tuple>

#include "kernels.h"
#include "rows.h"
#include "shard.h"

// Scratch of ss_decode_step_static: the buffers a decode step keeps between its kernels (residual
// rows, operand fragments, row sums, q|k|v, attention partials and counters, the LM head's
// candidates), for callers that cannot allocate.  Every device the library runs on holds its own
// copy of this array until the process ends; host code reaches it through the address
// hipGetSymbolAddress gives per device, never through the name.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace ss {

// ---------------------------------------------------------------------------
// row kernels
// ---------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) embed_rows(EmbedArgs a) {
  __shared__ float scratch[4];
  embed_row_block<T>(a, blockIdx.x, scratch);
}

// last prompt position of every sequence -> the decode step's residual rows, with the final
// norm's operand (x - c) * gamma, c the row's mean (RMSNorm: 0), the centred sums and c
template <typename T>
__global__ void __launch_bounds__(256) gather_last(const float *x, int S, float *xd, const float *gamma, void *act_out,
                                                   float *stat_out, float *cen_out, int d, int rms) {
  typedef typename Operand<T>::type OT;
  __shared__ float scratch[4];
  const int b = blockIdx.x;
  const float *src = x + ((size_t)b * S + S - 1) * d;
  float *dst = xd + (size_t)b * d;
  constexpr int PL = Elem<T>::kPerLane;
  float s1 = 0.f, s2 = 0.f;
  for (int k = threadIdx.x * PL; k < d; k += 256 * PL) {
#pragma unroll
    for (int e = 0; e < PL; ++e) {
      const float v = src[k + e];
      dst[k + e] = v;
      s1 += v;
    }
  }
  const float c = rms ? 0.f : block_sum(s1, scratch) / (float)d;
  s1 = 0.f;
  for (int k = threadIdx.x * PL; k < d; k += 256 * PL) {
    float y[PL];
#pragma unroll
    for (int e = 0; e < PL; ++e) {
      const float t = src[k + e] - c;
      s1 += t, s2 += t * t;
      y[e] = t * gamma[k + e];
    }
    store_piece<OT>(act_out, b, k, d / Elem<T>::kFragK, y);
  }
  s1 = block_sum(s1, scratch);
  s2 = block_sum(s2, scratch);
  if (threadIdx.x == 0) {
    ((f32x4 *)stat_out)[b] = f32x4{s1, s2, 0.f, 0.f};
    if (cen_out) cen_out[b] = c;
  }
}

// The last kernel of a step, one block per batch row: after an LM head, the greedy choice among
// the per-block candidates (highest logit, lowest index on ties: the result does not depend on
// the order they are looked at) -> next_tokens; then the token-level commit, n[b] += inc for every
// shard of the group: the last action of the step.  A stage that hands hidden states on has no
// candidates (am_val NULL) and only commits.
struct CommitArgs {
  const float *am_val;  // [32][n_blocks] or NULL
  const int *am_idx;
  int n_blocks;
  int32_t *next_tokens;  // [B] or NULL
  int32_t *lens[8];
  int cap[8];            // rows each shard's cache holds: a length never moves past it
  int n_lens, B, inc;
};
__global__ void __launch_bounds__(256) choose_and_commit(CommitArgs a) {
  __shared__ float s_v[256];
  __shared__ int s_i[256];
  const int row = blockIdx.x, tid = threadIdx.x;
  if (a.am_val && a.next_tokens) {
    float bv = -INFINITY;
    int bi = INT_MAX;
    const float *v = a.am_val + (size_t)row * a.n_blocks;
    const int *ix = a.am_idx + (size_t)row * a.n_blocks;
    constexpr int MB = 8;  // requests a thread makes in one go: the candidates come from memory, one round trip for 2048 blocks
    for (int g0 = tid; g0 < a.n_blocks; g0 += 256 * MB) {
      float ov[MB];
      int oi[MB];
#pragma unroll
      for (int i = 0; i < MB; ++i) {
        const int g = g0 + i * 256;
        const bool ok = g < a.n_blocks;
        ov[i] = ok ? v[g] : -INFINITY;
        oi[i] = ok ? ix[g] : INT_MAX;
      }
#pragma unroll
      for (int i = 0; i < MB; ++i)
        if (ov[i] > bv || (ov[i] == bv && oi[i] < bi)) bv = ov[i], bi = oi[i];
    }
    s_v[tid] = bv, s_i[tid] = bi;
    __syncthreads();
    for (int half = 128; half > 0; half >>= 1) {
      if (tid < half) {
        const float ov = s_v[tid + half];
        const int oi = s_i[tid + half];
        if (ov > s_v[tid] || (ov == s_v[tid] && oi < s_i[tid])) s_v[tid] = ov, s_i[tid] = oi;
      }
      __syncthreads();
    }
    if (tid == 0) a.next_tokens[row] = s_i[0];
  }
  if (tid == 0)
    for (int q = 0; q < a.n_lens; ++q) a.lens[q][row] = min(a.lens[q][row] + a.inc, a.cap[q]);
}
static ss_status launch_commit(const StreamGemmArgs &g, hipStream_t st) {
  if (g.B < 1 || g.B > 32 || g.n_lens < 0 || g.n_lens > 8) SS_FAIL(SS_EINVAL, "commit: batch %d, %d shards", g.B, g.n_lens);
  CommitArgs c = {};
  c.am_val = g.am_val, c.am_idx = g.am_idx, c.n_blocks = g.n_blocks, c.next_tokens = g.next_tokens;
  c.n_lens = g.n_lens, c.B = g.B, c.inc = g.commit_inc;
  for (int q = 0; q < c.n_lens; ++q) c.lens[q] = g.lens[q], c.cap[q] = g.len_cap[q];
  SS_LAUNCH_KERNEL(choose_and_commit, dim3(g.B), dim3(256), 0, st, c);
  SS_HIP(hipGetLastError());
  return SS_OK;
}

// ---------------------------------------------------------------------------
// group checks
// ---------------------------------------------------------------------------
static ss_status check_group(Shard *const *group, int n_group, int B) {
  if (!group || n_group < 1 || n_group > 8) SS_FAIL(SS_EINVAL, "group must hold 1..8 shards");
  for (int i = 0; i < n_group; ++i)
    if (!group[i]) SS_FAIL(SS_EINVAL, "group[%d] is NULL", i);
  const Shard *g0 = group[0];
  if (B < 1 || B > g0->L.Bmax) SS_FAIL(SS_EINVAL, "batch %d outside [1,%d]", B, g0->L.Bmax);
  for (int i = 1; i < n_group; ++i) {
    const Shard *s = group[i];
    if (s->s.layer_lo != g0->s.layer_lo || s->s.layer_hi != g0->s.layer_hi)
      SS_FAIL(SS_EINVAL, "shards of a group must hold the same layers");
    if (s->m.d_model != g0->m.d_model || s->m.head_dim != g0->m.head_dim || s->m.dtype != g0->m.dtype ||
        s->m.act != g0->m.act || s->m.pos != g0->m.pos || s->m.norm != g0->m.norm || s->m.kv_dtype != g0->m.kv_dtype)
      SS_FAIL(SS_EINVAL, "shards of a group must come from the same model");
    if (B > s->L.Bmax) SS_FAIL(SS_EINVAL, "batch %d exceeds group[%d]'s max_batch %d", B, i, s->L.Bmax);
    for (int j = 0; j < i; ++j) {
      const Shard *o = group[j];
      if (s == o) SS_FAIL(SS_EINVAL, "a shard appears twice in the group");
      if (s->s.head_lo < o->s.head_hi && o->s.head_lo < s->s.head_hi) SS_FAIL(SS_EINVAL, "head slices of the group overlap");
      if (s->s.ffn_lo < o->s.ffn_hi && o->s.ffn_lo < s->s.ffn_hi) SS_FAIL(SS_EINVAL, "FFN slices of the group overlap");
    }
  }
  return SS_OK;
}

static void attn_plan(const Layout &L, int B, int *rows_per_block, int *splits, int *waves) {
  const int pairs = std::max(1, B * L.Hs);
  // whole pairs pay off from 64 pairs on, unless the last round of blocks would leave most of the 256 compute
  // units idle
  const int rounds = ceil_div(pairs, 256);
  if (pairs >= 64 && (rounds == 1 || pairs * 4 >= rounds * 256 * 3)) {
    // one block per pair, merged in LDS: nothing of the softmax goes through memory.  Up to 256 pairs: 16 waves, a
    // compute unit to a block.  Between one and two pairs a unit: 8 waves, two blocks sharing a unit at the same time
    // (all pairs in one round; LLaMA-30B shape, 416 pairs: 37.8 us against 39.5 us for two rounds of 16-wave blocks).
    *rows_per_block = (int)align_up((size_t)L.Smax, 64), *splits = 1, *waves = rounds == 2 ? 8 : 16;
    return;
  }
  // few pairs: split the sequence over blocks of 4 waves (at least 64 rows each; the partial
  // buffer holds ceil(Smax/64) splits), the last block to arrive for a pair merges
  const int want = std::max(1, std::min(ceil_div(1024, pairs), L.attn_splits));
  const int rpb = (int)align_up((size_t)ceil_div(L.Smax, want), 64);
  *rows_per_block = rpb;
  *splits = ceil_div(L.Smax, rpb);
  *waves = 4;
}

// ---------------------------------------------------------------------------
// the decode step as a list of phases
// ---------------------------------------------------------------------------
// ---------------------------------------------------------------------------
// Launch shape of a decode GEMM: the kernel instance (weight tiles per block at most), the number
// of blocks the tiles are shared out over and, for the q|k|v GEMM, the slices K is cut into.  None
// of the first two changes a single bit of the result (the order of every sum is the same), so the
// choice is free; it is made per shape by a small cost model fitted to what this device shows
// (kernel-class timings inside decode steps of the three large shards, a dozen shapes each):
//  - a compute unit takes in about 45 GB/s whatever the source (weights from HBM, activation
//    fragments from L2), so with at most one block a unit the largest block decides; a block reads
//    its activation fragments once for all its tiles: more tiles a block, fewer bytes a unit;
//  - a long stream from HBM runs at about 6.8 TB/s;
//  - a kernel takes about the 6-norm of the two (near-equal bounds cost more than either);
//  - at equal largest block, more blocks are slower (about 0.09 % of the HBM time per block), so
//    an uneven share-out over all units loses to fewer blocks of one size;
//  - with several rounds of blocks, instances that fit twice on a unit (up to 2 tiles a block for
//    up to 16 batch rows, 1 tile above) stream about 15 % faster than the others, and the last
//    round costs about half a block;
//  - partial q|k|v sums cost the attention kernel that adds them a microsecond or two.
// ---------------------------------------------------------------------------
struct GemmShape {
  int nw, n_blocks, k_split;
  double est_us;  // the rule's estimate of the streaming time
};
struct ShapeKey {
  int epi, row_tiles, k_blocks, B, ks, split_max, split_cost_x10, forced_nw, forced_split, stat_groups;
  bool operator<(const ShapeKey &o) const {
    return std::tie(epi, row_tiles, k_blocks, B, ks, split_max, split_cost_x10, forced_nw, forced_split, stat_groups) <
           std::tie(o.epi, o.row_tiles, o.k_blocks, o.B, o.ks, o.split_max, o.split_cost_x10, o.forced_nw, o.forced_split, o.stat_groups);
  }
};
static std::map<ShapeKey, GemmShape> g_shapes;
static std::mutex g_shape_mu;
static std::atomic<uint64_t> g_shape_epoch{0};  // bumped when a forced shape changes what a plan would hold
static std::atomic<uint64_t> g_next_id{1};
uint64_t next_shard_id() { return g_next_id.fetch_add(1); }
static int g_forced_nw = 0, g_forced_split = 0;  // test aids: 0 = the rule's choice
static int forced_k_slices() {
  std::lock_guard<std::mutex> lock(g_shape_mu);
  return g_forced_split;
}

constexpr int kComputeUnits = 256;
constexpr double kUnitKiBPerUs = 45.0e9 / 1024.0 / 1.0e6;   // what one compute unit takes in
constexpr double kHbmKiBPerUs = 6.8e12 / 1024.0 / 1.0e6;    // a long stream from HBM

// estimated microseconds of streaming (without the few microseconds every launch costs); two_fit: two blocks of the instance fit on a unit
static double shape_cost(int tu, int units, int k_blocks, double act, double stat_kib, bool two_fit, int n_blocks, int S, double split_cost,
                         double unit_rate = 1.0) {
  const int upb = ceil_div(units, n_blocks);                  // units of the largest block
  const double kslice = (double)ceil_div(k_blocks, S);
  const int blocks = n_blocks * S;
  const double largest = ((double)upb * tu + act) * kslice + stat_kib;   // KiB the largest block takes in
  double t_cu;
  if (blocks <= kComputeUnits) {
    t_cu = largest / (kUnitKiBPerUs * unit_rate);
  } else if (act >= 2.0) {
    // More than 16 batch rows (one block a unit at a time, every block bound by the unit's intake): the blocks run in
    // rounds of 256, and a round takes what its largest block takes; a few blocks over a multiple of 256 cost a whole
    // round (measured on the OPT-66B shape's LM head: 524 blocks of 6 tiles took as long as 1048 of 3).  The blocks
    // with one unit more come first, so only the first rounds hold them.
    const int rounds = ceil_div(blocks, kComputeUnits), big = units % n_blocks == 0 ? blocks : (units % n_blocks) * S;
    const double smaller = ((double)(units / n_blocks) * tu + act) * kslice + stat_kib;
    t_cu = 0.0;
    for (int r = 0; r < rounds; ++r) t_cu += (r * kComputeUnits < big ? largest : smaller) / (kUnitKiBPerUs * unit_rate);
  } else {
    const double total = ((double)units * tu + (double)n_blocks * act) * k_blocks + (double)blocks * stat_kib;  // KiB all blocks take in
    t_cu = total / (kComputeUnits * kUnitKiBPerUs) * (two_fit ? 1.0 : 1.15) + 0.5 * largest / kUnitKiBPerUs;
  }
  const double t_hbm = (double)units * tu * k_blocks / kHbmKiBPerUs;
  const double norm6 = std::pow(std::pow(t_cu, 6.0) + std::pow(t_hbm, 6.0), 1.0 / 6.0);
  return norm6 + 0.00086 * t_hbm * std::min(blocks, kComputeUnits) + (S > 1 ? split_cost + 0.3 * (S - 2) : 0.0);
}

static GemmShape shape_rule(int epi, int row_tiles, int k_blocks, int B, int ks, int split_max, double split_cost,
                            int forced_nw, int forced_split, int stat_groups) {
  const int tu = epi == EPI_SWIGLU ? 2 : 1, units = row_tiles / tu;
  const double act = B <= 8 ? 0.5 : (B <= 16 ? 1.0 : 2.0);   // KiB of activation fragments per k block a block reads
  // six tiles a block: gate/up pairs and float output for up to 16 rows; for more rows float output only where the block adds
  // up no row statistics (that instance has no registers left to request them early), and the logits (a kernel long
  // enough not to mind)
  const bool wide = B <= 16 ? (epi == EPI_F32 || epi == EPI_SWIGLU) : ((epi == EPI_F32 && stat_groups == 0) || epi == EPI_LOGITS);
  // KiB of the producer's partial row sums every block of a normalised GEMM reads (a float4 per pair of weight tiles and
  // row): counted for more than 16 rows, where they reach 147 KiB a block on the OPT-66B shape; the constants for up to
  // 16 rows were fitted with them inside
  const double stat_kib = B > 16 ? (double)stat_groups * B * 16.0 / 1024.0 : 0.0;
  std::vector<int> instances;
  if (epi == EPI_SWIGLU) instances = {2};
  else instances = {1, 2, 3};
  if (wide) instances.push_back(6);
  if (forced_nw) {  // the nearest instance this GEMM has
    int nw = forced_nw;
    if (epi == EPI_SWIGLU) nw = (forced_nw >= 6 && wide) ? 6 : 2;
    else if (nw > 3) nw = (nw == 6 && wide) ? 6 : 3;
    instances = {nw};
  }
  GemmShape best = {0, 0, 1, 0.0};
  double best_t = 0;
  for (int S = 1; S <= std::max(1, split_max); ++S) {
    if (forced_split && S != forced_split) continue;
    if (S > 1 && k_blocks < S * ks) continue;
    for (int nw : instances) {
      const int upb_max = nw / tu;
      const bool two_fit = B <= 16 ? nw <= 2 : nw <= 1;
      // the six-tile instance for two batch tiles runs with every register taken: at equal bytes a block of it streams
      // about a tenth slower than a three-tile block (q|k|v of the OPT-66B shape: 16.5 us in 6-tile blocks x 5 slices,
      // 15.6 us in 3-tile blocks x 3 slices, 464 and 480 KiB a block)
      const double unit_rate = (B > 16 && nw == 6) ? 0.89 : 1.0;
      // block counts worth a look: the fewest for every size of the largest block (with a forced instance: its full size only)
      for (int upb = upb_max; upb >= 1; --upb) {
        const int n_blocks = ceil_div(units, upb);
        if (ceil_div(units, n_blocks) != upb) continue;       // the same share-out as a smaller size
        const double t = shape_cost(tu, units, k_blocks, act, stat_kib, two_fit, n_blocks, S, split_cost, unit_rate);
        if (!best.nw || t < best_t) best = {nw, n_blocks, S, t}, best_t = t;
        if (forced_nw) break;
      }
      // more than 16 rows and several rounds: block counts that fill whole rounds
      if (B > 16 && !forced_nw && S == 1) {
        for (int n_blocks = 2 * kComputeUnits; n_blocks <= units; n_blocks += kComputeUnits) {
          if (ceil_div(units, n_blocks) > upb_max) continue;
          const double t = shape_cost(tu, units, k_blocks, act, stat_kib, two_fit, n_blocks, S, split_cost, unit_rate);
          if (!best.nw || t < best_t) best = {nw, n_blocks, S, t}, best_t = t;
        }
      }
    }
  }
  if (!best.nw) best = {epi == EPI_SWIGLU ? 2 : 1, units, 1, 0.0};
  return best;
}

// fills in the launch shape; returns the rule's estimate of the streaming time (us)
static double shape_gemm(StreamGemmArgs &a, int epi) {
  const int split_max = (epi == EPI_F32 && a.split_ok > 1) ? std::min(a.split_ok, 8) : 1;
  GemmShape v;
  {
    std::lock_guard<std::mutex> lock(g_shape_mu);
    const int forced_split = std::min(g_forced_split, split_max);
    const ShapeKey key{epi, a.row_tiles, a.k_blocks, a.B, a.ks, split_max, (int)(a.split_cost_us * 10.f), g_forced_nw, forced_split, a.stat_groups};
    auto it = g_shapes.find(key);
    if (it == g_shapes.end())
      it = g_shapes.emplace(key, shape_rule(epi, a.row_tiles, a.k_blocks, a.B, a.ks, split_max, a.split_cost_us, g_forced_nw, forced_split, a.stat_groups)).first;
    v = it->second;
  }
  a.nw = v.nw, a.n_blocks = v.n_blocks, a.k_split = v.k_split;
  {
    const int units = epi == EPI_SWIGLU ? a.row_tiles / 2 : a.row_tiles;
    a.u_base = units / a.n_blocks, a.u_rem = units % a.n_blocks, a.k_slice = ceil_div(a.k_blocks, std::max(1, a.k_split));
  }
  a.part_stride = v.k_split > 1 ? (size_t)32 * a.ld_out : 0;
  return v.est_us;
}
static int pick_ks(int k_blocks) { return k_blocks >= 16 ? 8 : 4; }  // waves per block

// the final norm and the LM head over the rows in the decode buffers, greedy choice, commit
static Phase lm_head_phase(Shard *const *group, int n_group, int B, int stat_groups, float *logits, int32_t *next_tokens,
                           int commit_inc) {
  Shard *g0 = group[0];
  const Layout &L = g0->L;
  Phase ph = {};
  ph.kind = PH_LM_HEAD;
  StreamGemmArgs &a = ph.g;
  a.zero_frag = g0->zero_frag;
  a.w = g0->lm_head.ptr, a.row_tiles = g0->lm_head.row_tiles, a.k_blocks = g0->lm_head.k_blocks, a.B = B, a.N = L.V;
  a.ks = pick_ks(a.k_blocks);
  a.act = g0->dec_at(L.ws_ad);
  a.stat_in = (const float *)(g0->dec_at(L.ws_statd)), a.stat_groups = stat_groups, a.norm_dim = L.d;
  a.rms = g0->m.norm == SS_NORM_RMSNORM, a.eps = g0->m.norm_eps;
  a.wg = g0->wg_lm, a.cb = g0->cb_lm;
  a.out_f32 = logits, a.ld_out = L.V;
  a.am_val = (float *)(g0->dec_at(L.ws_argmax));
  a.next_tokens = next_tokens;
  for (int i = 0; i < n_group; ++i) a.lens[i] = group[i]->d_len, a.len_cap[i] = group[i]->L.Smax;
  a.n_lens = n_group, a.commit_inc = commit_inc;
  shape_gemm(a, EPI_LOGITS);
  a.am_idx = (int *)(a.am_val + (size_t)32 * a.n_blocks);  // [32][n_blocks] values, then as many indices
  ph.gx = a.n_blocks, ph.gy = 1;
  return ph;
}

// Phases of one decode step, in order.  The residual stream x, the operand of the next normalised
// GEMM (x * gamma) and the rows' partial sums live in group[0]'s workspace; q|k|v, the attention
// output and the FFN activation in each shard's own.
// Pipeline stages: hidden_in replaces the token lookup, hidden_out the final norm + LM head (the
// stage then commits with a kernel of its own).
static void build_decode_plan(Shard *const *group, int n_group, const int32_t *tokens_in, const float *hidden_in, int B,
                              float *hidden_out, float *logits, int32_t *next_tokens, int stop_after_layer,
                              std::vector<Phase> *plan) {
  Shard *g0 = group[0];
  const Layout &L0 = g0->L;
  const ss_model_desc &m = g0->m;
  const int dt = m.dtype, d = L0.d;
  const int FK = dt == SS_DTYPE_BF16 ? 32 : 16;
  const int rms = m.norm == SS_NORM_RMSNORM;
  float *x = (float *)(g0->dec_at(L0.ws_xd));
  void *ad = g0->dec_at(L0.ws_ad);
  float *statd = (float *)(g0->dec_at(L0.ws_statd));
  float *cen = rms ? nullptr : (float *)(g0->dec_at(L0.ws_cen));  // the rows' means at the last norm: centres of the next operand
  const float *first_gamma = g0->layers[0].ln1_g;
  plan->clear();
  {
    Phase ph = {};
    ph.kind = PH_EMBED, ph.gx = B, ph.gy = 1;
    ph.e = EmbedArgs{hidden_in, tokens_in, g0->wte, g0->wpe, g0->d_len, 0, L0.max_pos, x, d, L0.V, first_gamma, ad, nullptr, rms, statd, cen};
    plan->push_back(ph);
  }
  int stat_groups = 1;  // partial-sum groups behind the rows in statd
  // a GEMM whose input is Norm(x): operand x * gamma from the producer of x, statistics deferred
  auto normed = [&](StreamGemmArgs &a, const float *wg, const float *cb, int shard) {
    a.act = ad, a.stat_in = statd, a.stat_groups = stat_groups, a.norm_dim = d, a.rms = rms, a.eps = m.norm_eps;
    a.wg = wg, a.cb = cb;
    if (shard == 0) a.cen = cen, a.publish = 1;  // one consumer leaves the new mean for the next producer
  };
  // sum over the group at a reduce slot: shard i adds its partial to what the previous shards
  // left; the last one also emits the next operand (x * next_gamma) and the partial sums
  auto resid = [&](int i, const FragMat &w, const void *act, const float *bias, const float *next_gamma,
                   float *x_final) {
    Phase ph = {};
    ph.kind = PH_RESID, ph.shard = i;
    StreamGemmArgs &a = ph.g;
    a.zero_frag = g0->zero_frag;
    a.w = w.ptr, a.row_tiles = w.row_tiles, a.k_blocks = w.k_blocks, a.ks = pick_ks(a.k_blocks), a.B = B, a.N = d;
    a.act = act;
    a.cb = i == 0 ? bias : nullptr;
    a.x_in = x, a.x_out = x;
    if (i == n_group - 1) {
      if (x_final) a.x_out = x_final;  // the stage's output: no next GEMM in this shard
      else a.act_out = ad, a.out_k_blocks = d / FK, a.g_out = next_gamma, a.stat_out = statd, a.cen = cen;
    }
    shape_gemm(a, EPI_RESID);
    ph.gx = a.n_blocks, ph.gy = 1;
    plan->push_back(ph);
  };
  int qkv_parts[8] = {0};     // per shard of the group: partial q|k|v sums its GEMM leaves and their distance (floats)
  size_t qkv_stride[8] = {0};
  DecodeAttnArgs qkv_norm[8];  // and, where its GEMM leaves raw products, the normalisation the attention kernel applies
  for (int l = 0; l < L0.Ls; ++l) {
    const LayerDev &D0 = g0->layers[l];
    for (int i = 0; i < n_group; ++i) {  // QKV projection of the new token
      Shard *s = group[i];
      const Layout &L = s->L;
      Phase ph = {};
      ph.kind = PH_QKV, ph.shard = i;
      StreamGemmArgs &a = ph.g;
      a.zero_frag = s->zero_frag;
      a.w = s->wqkv[l].ptr, a.row_tiles = s->wqkv[l].row_tiles, a.k_blocks = s->wqkv[l].k_blocks, a.B = B, a.N = L.qkv_n;
      a.ks = pick_ks(a.k_blocks);
      normed(a, s->wg_qkv[l], s->cb_qkv[l], i);
      a.out_f32 = (float *)(s->dec_at(L.ws_qkvd)), a.ld_out = L.qkv_n;
      a.split_ok = kQkvParts;  // the consumer (decode attention) adds up to that many partial sums,
      a.split_cost_us = m.pos == SS_POS_ROPE ? 2.5f : 1.0f;  // which costs it this much (more where it rotates q and k: measured)
      // More than 16 batch rows: the GEMM leaves raw products and the attention kernel, which adds the slices up anyway,
      // applies the normalisation to the elements it stages.  The GEMM's blocks then read no row sums (147 KB each at
      // d = 9216 and 32 rows) and may be six tiles wide.
      qkv_norm[i] = DecodeAttnArgs{};
      if (B > 16) {
        DecodeAttnArgs &n = qkv_norm[i];
        n.stat_in = a.stat_in, n.stat_groups = a.stat_groups, n.norm_dim = a.norm_dim, n.rms = a.rms, n.eps = a.eps;
        n.wg = a.wg, n.cb = a.cb, n.cen = a.cen, n.publish = a.publish;
        a.stat_in = nullptr, a.stat_groups = 0, a.wg = nullptr, a.cb = nullptr, a.cen = nullptr, a.publish = 0;
      }
      shape_gemm(a, EPI_F32);
      ph.gx = a.n_blocks * a.k_split, ph.gy = 1;
      qkv_parts[i] = a.k_split, qkv_stride[i] = a.part_stride;
      plan->push_back(ph);
    }
    for (int i = 0; i < n_group; ++i) {  // attention over the committed rows + append
      Shard *s = group[i];
      const Layout &L = s->L;
      Phase ph = {};
      ph.kind = PH_ATTN, ph.shard = i;
      DecodeAttnArgs &a = ph.at;
      a.qkv = (const float *)(s->dec_at(L.ws_qkvd));
      a.qkv_parts = qkv_parts[i], a.qkv_stride = qkv_stride[i];
      {
        const DecodeAttnArgs &n = qkv_norm[i];
        a.stat_in = n.stat_in, a.stat_groups = n.stat_groups, a.norm_dim = n.norm_dim, a.rms = n.rms, a.eps = n.eps;
        a.wg = n.wg, a.cb = n.cb, a.cen = n.cen, a.publish = n.publish;
      }
      a.k_cache = s->kv_ptr(l, 0), a.v_cache = s->kv_ptr(l, 1);
      a.row_stride = s->kv_row_stride(), a.head_stride = s->kv_head_stride();
      a.lens = s->d_len, a.rope = m.pos == SS_POS_ROPE ? s->rope : nullptr;
      a.part = (float *)(s->dec_at(L.ws_attn_part));
      a.counters = (int *)(s->dec_at(L.ws_counters)) + 16;
      a.o_out = s->dec_at(L.ws_od);
      a.B = B, a.Hs = L.Hs, a.Dh = L.Dh, a.Smax = L.Smax, a.kv_dtype = s->m.kv_dtype;
      attn_plan(L, B, &a.rows_per_block, &a.splits, &a.waves);
      ph.gx = B * L.Hs, ph.gy = a.splits;
      plan->push_back(ph);
    }
    stat_groups = d / 32;  // from here on the partial sums come from the residual GEMMs' weight tile pairs
    for (int i = 0; i < n_group; ++i)  // output projection, sum over the group, residual
      resid(i, group[i]->wo[l], group[i]->dec_at(group[i]->L.ws_od), D0.bo, D0.ln2_g, nullptr);
    for (int i = 0; i < n_group; ++i) {  // first FFN matrix + activation
      Shard *s = group[i];
      const Layout &L = s->L;
      Phase ph = {};
      ph.kind = PH_FFN_UP, ph.shard = i;
      StreamGemmArgs &a = ph.g;
      a.zero_frag = s->zero_frag;
      a.w = s->w1[l].ptr, a.row_tiles = s->w1[l].row_tiles, a.k_blocks = s->w1[l].k_blocks, a.B = B, a.N = L.Fs;
      a.ks = pick_ks(a.k_blocks);
      normed(a, s->wg_1[l], s->cb_1[l], i);
      a.act_out = s->dec_at(L.ws_ud), a.out_k_blocks = L.Fs / FK, a.act_kind = m.act;
      const double whole = shape_gemm(a, m.act == SS_ACT_SWIGLU ? EPI_SWIGLU : EPI_ACT);
      // More than 16 batch rows: every block reads two activation fragments per k block whatever its tiles, and
      // the tiles alone fill few compute units.  K in slices (float partial outputs, wide blocks) streams faster
      // and costs one more small kernel, which adds the slices up and applies the activation.
      if (B > 16 && L.ffnpart_bytes && m.act != SS_ACT_SWIGLU && forced_k_slices() != 1) {
        Phase cut = ph;
        StreamGemmArgs &c = cut.g;
        c.act_out = nullptr, c.out_k_blocks = 0;
        // raw partial products: the normalisation moves to the kernel that adds them up
        c.stat_in = nullptr, c.stat_groups = 0, c.wg = nullptr, c.cb = nullptr, c.cen = nullptr, c.publish = 0;
        c.out_f32 = (float *)(s->dec_at(L.ws_ffnpart)), c.ld_out = L.Fs;
        c.split_ok = kQkvParts, c.split_cost_us = 4.0f;  // the extra kernel
        const double sliced = shape_gemm(c, EPI_F32);
        if (c.k_split > 1 && (forced_k_slices() > 1 || sliced < whole)) {
          cut.gx = c.n_blocks * c.k_split, cut.gy = 1, cut.epi = EPI_F32;
          plan->push_back(cut);
          Phase fx = {};
          fx.kind = PH_FFN_ACT, fx.shard = i;
          StreamGemmArgs &f = fx.g;
          f.B = B, f.N = L.Fs, f.out_f32 = c.out_f32, f.ld_out = c.ld_out, f.k_split = c.k_split, f.part_stride = c.part_stride;
          f.act_out = a.act_out, f.out_k_blocks = a.out_k_blocks, f.act_kind = m.act;
          f.stat_in = a.stat_in, f.stat_groups = a.stat_groups, f.norm_dim = a.norm_dim, f.rms = a.rms, f.eps = a.eps;
          f.wg = a.wg, f.cb = a.cb, f.cen = a.cen, f.publish = a.publish;
          fx.gx = act_fixup_blocks(f), fx.gy = B;
          plan->push_back(fx);
          continue;
        }
      }
      ph.gx = a.n_blocks, ph.gy = 1, ph.epi = m.act == SS_ACT_SWIGLU ? EPI_SWIGLU : EPI_ACT;
      plan->push_back(ph);
    }
    const float *next_gamma = l + 1 < L0.Ls ? g0->layers[l + 1].ln1_g : g0->lnf_g;
    for (int i = 0; i < n_group; ++i)  // second FFN matrix, sum over the group, residual
      resid(i, group[i]->w2[l], group[i]->dec_at(group[i]->L.ws_ud), D0.b2, next_gamma,
            l + 1 == L0.Ls ? hidden_out : nullptr);
    if (l == stop_after_layer) return;
  }
  if (hidden_out) {
    Phase ph = {};
    ph.kind = PH_COMMIT, ph.gx = B, ph.gy = 1;
    ph.g.B = B, ph.g.n_lens = n_group, ph.g.commit_inc = 1;
    for (int i = 0; i < n_group; ++i) ph.g.lens[i] = group[i]->d_len, ph.g.len_cap[i] = group[i]->L.Smax;
    plan->push_back(ph);
    return;
  }
  Phase lm = lm_head_phase(group, n_group, B, stat_groups, logits, next_tokens, 1);
  plan->push_back(lm);
  lm.kind = PH_COMMIT, lm.gx = B, lm.gy = 1;  // picks the tokens among the LM head's candidates, then commits
  plan->push_back(lm);
}

// ---------------------------------------------------------------------------
// measurement aid: the next launch records its begin and end on a pair of the shard's events
// ---------------------------------------------------------------------------
thread_local LaunchTiming g_launch_timing;

struct Bracket {
  Shard *sh;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int cls;
  static hipEvent_t get(Shard *sh) {
    if (!sh->free_events.empty()) {
      hipEvent_t e = sh->free_events.back();
      sh->free_events.pop_back();
      return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
  Bracket(Shard *s, int c) : sh(s), cls(c) {
    if (!sh->timing) return;
    e0 = get(sh), e1 = get(sh);
    if (e0 && e1) g_launch_timing.start = e0, g_launch_timing.stop = e1;
  }
  ~Bracket() {
    g_launch_timing = LaunchTiming();
    if (!sh->timing || !e0 || !e1) return;
    sh->timed.push_back({cls, e0, e1});
  }
};

// one phase as a kernel of its own
static ss_status launch_phase(Shard *g0, const Phase &ph, hipStream_t st) {
  const int dt = g0->m.dtype;
  Bracket br(g0, ph.kind == PH_FFN_ACT ? (int)PH_FFN_UP : ph.kind);  // the sliced first FFN matrix and its activation kernel are one class
  switch (ph.kind) {
    case PH_EMBED:
      if (dt == SS_DTYPE_BF16) SS_LAUNCH_KERNEL(embed_rows<bf16_t>, dim3(ph.gx), dim3(256), 0, st, ph.e);
      else SS_LAUNCH_KERNEL(embed_rows<float>, dim3(ph.gx), dim3(256), 0, st, ph.e);
      SS_HIP(hipGetLastError());
      return SS_OK;
    case PH_QKV: return launch_stream_gemm(dt, EPI_F32, ph.g, st);
    case PH_ATTN: return launch_decode_attn(dt, ph.at, st);
    case PH_RESID: return launch_stream_gemm(dt, EPI_RESID, ph.g, st);
    case PH_FFN_UP: return launch_stream_gemm(dt, ph.epi, ph.g, st);
    case PH_FFN_ACT: return launch_act_fixup(dt, ph.g, st);
    case PH_LM_HEAD: return launch_stream_gemm(dt, EPI_LOGITS, ph.g, st);
    case PH_COMMIT: return launch_commit(ph.g, st);
  }
  SS_FAIL(SS_EINVAL, "unknown phase kind %d", ph.kind);
}

static ss_status enqueue_decode(Shard *const *group, int n_group, const int32_t *tokens_in, const float *hidden_in, int B,
                                float *hidden_out, float *logits, int32_t *next_tokens, hipStream_t st,
                                int stop_after_layer) {
  static thread_local std::vector<Phase> plan;  // kept between steps: no host allocation after a thread's first step
  build_decode_plan(group, n_group, tokens_in, hidden_in, B, hidden_out, logits, next_tokens, stop_after_layer, &plan);
  for (const Phase &ph : plan) SS_TRY(launch_phase(group[0], ph, st));
  if (stop_after_layer >= 0)
    SS_FAIL(SS_EINTR, "decode step interrupted after layer %d; nothing committed", stop_after_layer);
  return SS_OK;
}

void destroy_graphs(Shard *sh) {
  for (auto &kv : sh->graphs) (void)hipGraphExecDestroy(kv.second);
  sh->graphs.clear();
  for (auto &t : sh->timed) (void)hipEventDestroy(t.e0), (void)hipEventDestroy(t.e1);
  sh->timed.clear();
  for (auto e : sh->free_events) (void)hipEventDestroy(e);
  sh->free_events.clear();
}

ss_status run_decode_step(Shard *const *group, int n_group, const int32_t *tokens_in, const float *hidden_in, int B,
                          float *hidden_out, float *logits, int32_t *next_tokens, hipStream_t st,
                          int stop_after_layer) {
  Shard *g0 = group[0];
  GraphKey key;
  key.B = B;
  key.epoch = g_shape_epoch.load();
  key.ptrs = {tokens_in, hidden_in, hidden_out, logits, next_tokens, (const void *)st};
  for (int i = 0; i < n_group; ++i) key.ids.push_back(group[i]->id);
  const bool plain = !g0->timing && stop_after_layer < 0;
  // the NULL stream cannot be captured, and a stream the caller is capturing is left to the caller
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  if (st) SS_HIP(hipStreamIsCapturing(st, &cs));
  const bool graph = g0->use_graph && plain && st != nullptr && cs == hipStreamCaptureStatusNone;
  if (!graph)
    return enqueue_decode(group, n_group, tokens_in, hidden_in, B, hidden_out, logits, next_tokens, st, stop_after_layer);
  auto it = g0->graphs.find(key);
  if (it == g0->graphs.end()) {
    hipGraph_t gr = nullptr;
    SS_HIP(hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
    ss_status rc = enqueue_decode(group, n_group, tokens_in, hidden_in, B, hidden_out, logits, next_tokens, st, -1);
    hipError_t e = hipStreamEndCapture(st, &gr);
    if (rc != SS_OK) {
      if (gr) (void)hipGraphDestroy(gr);
      return rc;
    }
    if (e != hipSuccess) SS_FAIL(SS_EHIP, "hipStreamEndCapture: %s", hipGetErrorString(e));
    hipGraphExec_t ex = nullptr;
    e = hipGraphInstantiate(&ex, gr, nullptr, nullptr, 0);
    (void)hipGraphDestroy(gr);
    if (e != hipSuccess) SS_FAIL(SS_EHIP, "hipGraphInstantiate: %s", hipGetErrorString(e));
    if (g0->graphs.size() >= 16) {  // rare: an exec may still be running on the stream it was launched on
      SS_HIP(hipStreamSynchronize(st));
      for (auto &kv : g0->graphs) (void)hipGraphExecDestroy(kv.second);
      g0->graphs.clear();
    }
    it = g0->graphs.emplace(key, ex).first;
  }
  SS_HIP(hipGraphLaunch(it->second, st));
  return SS_OK;
}

// ---------------------------------------------------------------------------
// the initial phase
// ---------------------------------------------------------------------------
ss_status run_prefill(Shard *const *group, int n_group, const int32_t *tokens, const float *hidden_in, int B, int S,
                      float *hidden_out, float *logits, int32_t *next_tokens, hipStream_t st) {
  Shard *g0 = group[0];
  const Layout &L0 = g0->L;
  const ss_model_desc &m = g0->m;
  const int dt = m.dtype, d = L0.d;
  const int FK = dt == SS_DTYPE_BF16 ? 32 : 16;
  const int rms = m.norm == SS_NORM_RMSNORM;
  const int T_live = B * S, T = (int)align_up((size_t)T_live, 256);
  for (int i = 0; i < n_group; ++i)
    if (T > group[i]->L.Tmax) SS_FAIL(SS_EINVAL, "%d prompt tokens exceed group[%d]'s workspace (%d)", T_live, i, group[i]->L.Tmax);
  float *x = (float *)(g0->ws + L0.ws_x);
  void *abuf = g0->ws + L0.ws_a;
  void *abuf_lo = L0.two_part_qk ? g0->ws + L0.ws_a_lo : nullptr;  // low parts of the q|k|v GEMM's operand
  float2 *pstat = (float2 *)(g0->ws + L0.ws_pstat);
  f32x4 *mr = (f32x4 *)(pstat + (size_t)2 * ceil_div(d, 128) * L0.Tmax);  // (mean, rstd, mean - centre, -) per token
  // Norms are deferred and centred (see TileGemmArgs): the producer of x writes (x - c) * gamma as the
  // next GEMM's operand and partial row sums; that GEMM's epilogue normalises.  Operands are halves
  // for bf16 models: single bf16 activations miss the logits bar (OPT-66B shape 6.4e-2 at its first
  // token), bf16 hi/lo pairs meet it at twice the matrix-core work.
  {
    EmbedArgs e{hidden_in, tokens, g0->wte, g0->wpe, nullptr, S, L0.max_pos, x, d, L0.V, g0->layers[0].ln1_g, abuf, abuf_lo, rms, nullptr, nullptr, pstat, mr};
    if (dt == SS_DTYPE_BF16) hipLaunchKernelGGL(embed_rows<bf16_t>, dim3(T_live), dim3(256), 0, st, e);
    else hipLaunchKernelGGL(embed_rows<float>, dim3(T_live), dim3(256), 0, st, e);
    SS_HIP(hipGetLastError());
  }
  int stat_groups = 1;
  auto normed = [&](TileGemmArgs &a, const float *wg, const float *cb) {
    a.act = abuf, a.mr_in = mr, a.wg = wg, a.cb = cb;
  };
  auto row_stats = [&]() { return launch_row_stats(pstat, stat_groups, T, d, rms, m.norm_eps, mr, st); };
  // sum over the group at a reduce slot: shard i adds its partial to what the previous shards left;
  // the last one also emits the next operand and the partial sums
  auto resid = [&](int i, const FragMat &w, const void *act, const float *bias, const float *next_gamma, bool feeds_qkv) -> ss_status {
    TileGemmArgs a = {};
    a.w = w.ptr, a.row_tiles = w.row_tiles, a.k_blocks = w.k_blocks;
    a.act = act, a.T = T, a.T_live = T_live, a.N = d, a.bias = i == 0 ? bias : nullptr;
    a.x_resid = x;
    if (i == n_group - 1 && next_gamma) {
      a.g_out = next_gamma, a.norm_out = abuf, a.stat_out = pstat, a.c_in = mr;
      if (feeds_qkv) a.norm_out_lo = abuf_lo;
    }
    return launch_tile_gemm(dt, EPI_RESID, a, st);
  };
  for (int l = 0; l < L0.Ls; ++l) {
    const LayerDev &D0 = g0->layers[l];
    SS_TRY(row_stats());
    for (int i = 0; i < n_group; ++i) {
      Shard *s = group[i];
      const Layout &L = s->L;
      TileGemmArgs a = {};
      a.w = s->wqkv[l].ptr, a.row_tiles = s->wqkv[l].row_tiles, a.k_blocks = s->wqkv[l].k_blocks;
      a.T = T, a.T_live = T_live, a.N = L.qkv_n;
      normed(a, s->wg_qkv[l], s->cb_qkv[l]);
      if (abuf_lo) a.act_lo = abuf_lo, a.lo_row_begin = 0, a.lo_row_end = 2 * L.Hs * L.Dh / 16;  // the q and k rows
      a.out_f32 = (float *)(s->ws + L.ws_qkv), a.ld_out = L.qkv_n;
      // The GEMM's epilogue writes the cache rows itself, rotating q and k first in a model with rotary positions where
      // its block shape holds whole heads per wave; otherwise a kernel of its own rotates and writes behind it.
      const bool rope_model = m.pos == SS_POS_ROPE;
      const bool gemm_rotates = rope_model && tile_gemm_rotates(dt, a, L.Dh);
      if (!rope_model || gemm_rotates) {
        a.k_cache = s->kv_ptr(l, 0), a.v_cache = s->kv_ptr(l, 1);
        a.kv_row_stride = s->kv_row_stride(), a.kv_head_stride = s->kv_head_stride();
        a.kv_S = S, a.kv_Hs = L.Hs, a.kv_Dh = L.Dh, a.kv_dtype = s->m.kv_dtype;
        if (gemm_rotates) a.rope = s->rope;
      }
      SS_TRY(launch_tile_gemm(dt, EPI_F32, a, st));
      PrefillAttnArgs p = {};
      p.qkv = (float *)(s->ws + L.ws_qkv);
      p.k_cache = s->kv_ptr(l, 0), p.v_cache = s->kv_ptr(l, 1);
      p.row_stride = s->kv_row_stride(), p.head_stride = s->kv_head_stride();
      p.rope = m.pos == SS_POS_ROPE ? s->rope : nullptr;
      p.o_out = s->ws + L.ws_o;
      p.B = B, p.S = S, p.Hs = L.Hs, p.Dh = L.Dh, p.Smax = L.Smax, p.kv_dtype = s->m.kv_dtype;
      p.vt = s->ws + L.ws_vt, p.s_pad = (int)align_up((size_t)S, 64);
      if (rope_model && !gemm_rotates) SS_TRY(launch_prefill_kv_write(dt, p, st));  // rotates q and k, writes the cache rows
      SS_TRY(launch_prefill_attn(dt, p, st));
    }
    stat_groups = 2 * ceil_div(d / 16, 8);  // from here on: one partial per 64-feature band of the residual GEMMs
    for (int i = 0; i < n_group; ++i) SS_TRY(resid(i, group[i]->wo[l], group[i]->ws + group[i]->L.ws_o, D0.bo, D0.ln2_g, false));
    SS_TRY(row_stats());
    for (int i = 0; i < n_group; ++i) {
      Shard *s = group[i];
      const Layout &L = s->L;
      const bool glu = m.act == SS_ACT_SWIGLU;
      TileGemmArgs a = {};
      a.w = s->w1[l].ptr, a.row_tiles = s->w1[l].row_tiles, a.k_blocks = s->w1[l].k_blocks;
      a.T = T, a.T_live = T_live, a.N = L.Fs;
      normed(a, s->wg_1[l], s->cb_1[l]);
      a.act_out = s->ws + L.ws_u, a.out_k_blocks = L.Fs / FK, a.act_kind = m.act;
      SS_TRY(launch_tile_gemm(dt, glu ? EPI_SWIGLU : EPI_ACT, a, st));
    }
    // the last layer's output goes to the next stage or to gather_last, which read x
    const float *next_gamma = l + 1 < L0.Ls ? g0->layers[l + 1].ln1_g : nullptr;
    for (int i = 0; i < n_group; ++i) SS_TRY(resid(i, group[i]->w2[l], group[i]->ws + group[i]->L.ws_u, D0.b2, next_gamma, true));
  }
  if (hidden_out) {  // a stage that hands its hidden states on: copy them out, then commit
    SS_HIP(hipMemcpyAsync(hidden_out, x, (size_t)T_live * d * 4, hipMemcpyDeviceToDevice, st));
    StreamGemmArgs c = {};
    c.n_lens = n_group, c.B = B, c.commit_inc = S;
    for (int i = 0; i < n_group; ++i) c.lens[i] = group[i]->d_len, c.len_cap[i] = group[i]->L.Smax;
    return launch_commit(c, st);
  }
  float *xd = (float *)(g0->dec_at(L0.ws_xd));
  void *ad = g0->dec_at(L0.ws_ad);
  float *statd = (float *)(g0->dec_at(L0.ws_statd));
  float *cen = rms ? nullptr : (float *)(g0->dec_at(L0.ws_cen));
  if (dt == SS_DTYPE_BF16) hipLaunchKernelGGL(gather_last<bf16_t>, dim3(B), dim3(256), 0, st, x, S, xd, g0->lnf_g, ad, statd, cen, d, rms);
  else hipLaunchKernelGGL(gather_last<float>, dim3(B), dim3(256), 0, st, x, S, xd, g0->lnf_g, ad, statd, cen, d, rms);
  SS_HIP(hipGetLastError());
  const Phase ph = lm_head_phase(group, n_group, B, 1, logits, next_tokens, S);
  SS_TRY(launch_stream_gemm(dt, EPI_LOGITS, ph.g, st));
  return launch_commit(ph.g, st);
}

}  // namespace ss

using namespace ss;

extern "C" {

static ss_status check_stage_io(const void *tokens, const void *hidden_in, const void *hidden_out, const void *logits,
                                const void *next_tokens) {
  if ((tokens != nullptr) == (hidden_in != nullptr)) SS_FAIL(SS_EINVAL, "give exactly one of tokens and hidden_in");
  if (hidden_out && (logits || next_tokens)) SS_FAIL(SS_EINVAL, "a stage with hidden_out produces no logits or tokens");
  return SS_OK;
}

ss_status ss_stage_prefill(ss_shard *const *group_, int32_t n_group, const int32_t *tokens, const float *hidden_in,
                           int32_t B, int32_t S_in, float *hidden_out, float *logits, int32_t *next_tokens,
                           void *hip_stream) {
  Shard *const *group = (Shard *const *)group_;
  SS_TRY(check_stage_io(tokens, hidden_in, hidden_out, logits, next_tokens));
  SS_TRY(check_group(group, n_group, B));
  if (S_in < 1) SS_FAIL(SS_EINVAL, "S_in must be positive");
  for (int i = 0; i < n_group; ++i) {
    if (S_in > group[i]->L.Smax) SS_FAIL(SS_EINVAL, "S_in %d exceeds group[%d]'s max_seq %d", S_in, i, group[i]->L.Smax);
    for (int b = 0; b < B; ++b)
      if (group[i]->h_len[b] != 0) SS_FAIL(SS_ESTATE, "row %d of group[%d] already holds %d tokens", b, i, group[i]->h_len[b]);
  }
  SS_TRY(run_prefill(group, n_group, tokens, hidden_in, B, S_in, hidden_out, logits, next_tokens, (hipStream_t)hip_stream));
  for (int i = 0; i < n_group; ++i)
    for (int b = 0; b < B; ++b) group[i]->h_len[b] = S_in;
  return SS_OK;
}

ss_status ss_prefill(ss_shard *const *group_, int32_t n_group, const int32_t *tokens, int32_t B, int32_t S_in,
                     float *logits, int32_t *next_tokens, void *hip_stream) {
  if (!tokens) SS_FAIL(SS_EINVAL, "tokens is NULL");
  return ss_stage_prefill(group_, n_group, tokens, nullptr, B, S_in, nullptr, logits, next_tokens, hip_stream);
}

// Host-only check aid: the phase table of one decode step for a shard of the given shape whose
// device memory starts at address `fake_base` (nothing is allocated or launched).  Writes up to
// max_phases Phase records to out_phases, the layout's total bytes to out_total, returns the
// number of phases (negative on error).
int32_t ss_debug_plan(const ss_model_desc *desc, const ss_slice *slice, int32_t max_batch, int32_t max_seq, int32_t B,
                      uint64_t fake_base, void *out_phases, int32_t max_phases, uint64_t *out_total,
                      uint64_t *out_sizeof_phase) {
  if (!desc || !slice || validate_desc(*desc, *slice, max_batch, max_seq) != SS_OK) return -1;
  Shard sh;
  sh.m = *desc, sh.s = *slice;
  compute_layout(*desc, *slice, max_batch, max_seq, &sh.L);
  const Layout &L = sh.L;
  sh.base = (char *)fake_base;
  bind_pointers(&sh);
  Shard *group[1] = {&sh};
  std::vector<Phase> plan;
  build_decode_plan(group, 1, (const int32_t *)8, nullptr, B, nullptr, (float *)16, (int32_t *)24, -1, &plan);
  if (out_total) *out_total = L.total;
  if (out_sizeof_phase) *out_sizeof_phase = sizeof(Phase);
  const int n = (int)plan.size();
  if (out_phases)
    for (int i = 0; i < n && i < max_phases; ++i) memcpy((char *)out_phases + (size_t)i * sizeof(Phase), &plan[i], sizeof(Phase));
  return n;
}

ss_status ss_debug_force_gemm_shape(int32_t tiles_per_block, int32_t k_slices) {
  if (tiles_per_block < 0 || tiles_per_block > 6 || k_slices < 0 || k_slices > 8)
    SS_FAIL(SS_EINVAL, "launch shape (%d, %d)", tiles_per_block, k_slices);
  std::lock_guard<std::mutex> lock(g_shape_mu);
  g_forced_nw = tiles_per_block, g_forced_split = k_slices;
  g_shape_epoch.fetch_add(1);
  return SS_OK;
}

ss_status ss_kernel_timing(ss_shard *shard, int32_t enabled) {
  if (!shard) SS_FAIL(SS_EINVAL, "NULL shard");
  ((Shard *)shard)->timing = enabled != 0;
  return SS_OK;
}

ss_status ss_kernel_timing_read(ss_shard *shard, double ms[8], int64_t count[8], void *hip_stream) {
  if (!shard || !ms || !count) SS_FAIL(SS_EINVAL, "NULL argument");
  Shard *sh = (Shard *)shard;
  SS_HIP(hipStreamSynchronize((hipStream_t)hip_stream));
  for (int i = 0; i < 8; ++i) ms[i] = 0.0, count[i] = 0;
  for (auto &t : sh->timed) {
    float f = 0.f;
    if (hipEventElapsedTime(&f, t.e0, t.e1) == hipSuccess && t.cls >= 0 && t.cls < 8) ms[t.cls] += f, count[t.cls] += 1;
    sh->free_events.push_back(t.e0);
    sh->free_events.push_back(t.e1);
  }
  sh->timed.clear();
  return SS_OK;
}

// what every decode-step entry point checks on the host before anything is launched
static ss_status check_decode_state(Shard *const *group, int n_group, int B) {
  SS_TRY(check_group(group, n_group, B));
  for (int b = 0; b < B; ++b) {
    const int n = group[0]->h_len[b];
    for (int i = 0; i < n_group; ++i) {
      if (group[i]->h_len[b] != n)
        SS_FAIL(SS_ESTATE, "row %d: group[%d] committed %d tokens, group[0] %d", b, i, group[i]->h_len[b], n);
      if (n + 1 > group[i]->L.Smax) SS_FAIL(SS_ESTATE, "row %d: cache of group[%d] is full (%d rows)", b, i, n);
    }
  }
  return SS_OK;
}

ss_status ss_stage_decode_step(ss_shard *const *group_, int32_t n_group, const int32_t *tokens_in, const float *hidden_in,
                               int32_t B, float *hidden_out, float *logits, int32_t *next_tokens, void *hip_stream) {
  Shard *const *group = (Shard *const *)group_;
  SS_TRY(check_stage_io(tokens_in, hidden_in, hidden_out, logits, next_tokens));
  SS_TRY(check_decode_state(group, n_group, B));
  int stop = -1;
  for (int i = 0; i < n_group; ++i) stop = std::max(stop, group[i]->interrupt_after);
  ss_status rc = run_decode_step(group, n_group, tokens_in, hidden_in, B, hidden_out, logits, next_tokens,
                                 (hipStream_t)hip_stream, stop);
  if (rc != SS_OK) return rc;  // SS_EINTR: nothing committed
  for (int i = 0; i < n_group; ++i)
    for (int b = 0; b < B; ++b) group[i]->h_len[b] += 1;
  return SS_OK;
}

ss_status ss_decode_step(ss_shard *const *group_, int32_t n_group, const int32_t *tokens_in, int32_t B, float *logits,
                         int32_t *next_tokens, void *hip_stream) {
  if (!tokens_in) SS_FAIL(SS_EINVAL, "tokens_in is NULL");
  return ss_stage_decode_step(group_, n_group, tokens_in, nullptr, B, nullptr, logits, next_tokens, hip_stream);
}

// ---------------------------------------------------------------------------
// The decode step for callers that cannot allocate: the step's scratch is the static device
// array `scratch` instead of the shards' workspaces, the kernels are launched one by one (a graph
// would have to be instantiated), and nothing is allocated on the device.
// ---------------------------------------------------------------------------
__global__ void zero_i32(int32_t *p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

constexpr int kMaxDevices = 64;
static char *g_scratch_ptr[kMaxDevices];  // the device address of `scratch` on each device
static std::mutex g_scratch_mu;

size_t ss_static_scratch_bytes(void) { return kStaticScratchBytes; }

ss_status ss_decode_step_static(ss_shard *const *group_, int32_t n_group, const int32_t *tokens_in, int32_t B,
                                float *logits, int32_t *next_tokens, void *hip_stream) {
  if (!tokens_in) SS_FAIL(SS_EINVAL, "tokens_in is NULL");
  Shard *const *group = (Shard *const *)group_;
  SS_TRY(check_decode_state(group, n_group, B));
  for (int i = 0; i < n_group; ++i)
    if (group[i]->timing) SS_FAIL(SS_ESTATE, "kernel timing is on for group[%d]: its events would have to be created", i);
  // this device's copy of the array (looked up once per device, with the device current)
  int dev = -1;
  SS_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) SS_FAIL(SS_EINVAL, "device %d outside [0,%d)", dev, kMaxDevices);
  char *base = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
      void *p = nullptr;
      SS_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
      if (!p) SS_FAIL(SS_EHIP, "hipGetSymbolAddress gave no address for the static scratch");
      g_scratch_ptr[dev] = (char *)p;
    }
    base = g_scratch_ptr[dev];
  }
  // every shard of the group gets its slice of the array
  size_t offs[8], total = 0;
  for (int i = 0; i < n_group; ++i) {
    offs[i] = total;
    total += align_up(group[i]->L.ws_dec_end - group[i]->L.ws_xd, 256);
  }
  if (total > kStaticScratchBytes)
    SS_FAIL(SS_ENOMEM, "a decode step of this group needs %zu bytes of scratch, the static array holds %zu", total,
            kStaticScratchBytes);
  hipStream_t st = (hipStream_t)hip_stream;
  char *saved[8];
  for (int i = 0; i < n_group; ++i) saved[i] = group[i]->dec, group[i]->dec = base + offs[i];
  ss_status rc = SS_OK;
  // the array keeps the last call's bytes: the attention kernels' arrival counters must start at zero
  for (int i = 0; i < n_group && rc == SS_OK; ++i) {
    const int nc = group[i]->L.n_counters;
    hipLaunchKernelGGL(zero_i32, dim3(ceil_div(nc, 256)), dim3(256), 0, st, (int32_t *)group[i]->dec_at(group[i]->L.ws_counters), nc);
    if (hipGetLastError() != hipSuccess) set_error("clearing the static scratch's counters failed"), rc = SS_EHIP;
  }
  int stop = -1;
  for (int i = 0; i < n_group; ++i) stop = std::max(stop, group[i]->interrupt_after);
  if (rc == SS_OK) rc = enqueue_decode(group, n_group, tokens_in, nullptr, B, nullptr, logits, next_tokens, st, stop);
  for (int i = 0; i < n_group; ++i) group[i]->dec = saved[i];
  if (rc != SS_OK) return rc;  // SS_EINTR: nothing committed
  for (int i = 0; i < n_group; ++i)
    for (int b = 0; b < B; ++b) group[i]->h_len[b] += 1;
  return SS_OK;
}

}  // extern "C"
