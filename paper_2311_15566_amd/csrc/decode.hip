// The decode step and the initial phase: row kernels (embedding, norms) and the launch
// sequence over a group of co-resident shards, with HIP-graph replay of the decode step.
#include <stdlib.h>
#include <string.h>

#include <algorithm>

#include "kernels.h"
#include "rows.h"
#include "shard.h"

namespace ss {

// ---------------------------------------------------------------------------
// row kernels
// ---------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) embed_rows(EmbedArgs a) {
  __shared__ float scratch[4];
  embed_row_block<T, true>(a, blockIdx.x, scratch);
}

// a = Norm(x) for every token row, written in operand order.  grid = rows.
template <typename T>
__global__ void __launch_bounds__(256) norm_rows(const float *x, const float *gamma, const float *beta, void *a_out,
                                                 int d, int k_blocks, int rms, float eps) {
  __shared__ float scratch[4];
  const int r = blockIdx.x;
  const float *xr = x + (size_t)r * d;
  float mean, rstd;
  row_stats(xr, d, rms, eps, scratch, &mean, &rstd);
  for (int k = threadIdx.x; k < d; k += 256) {
    float y = (xr[k] - mean) * rstd * gamma[k];
    if (beta) y += beta[k];
    store_act<T>(a_out, r, k, k_blocks, Elem<T>::kParts, y);
  }
}

// last prompt position of every sequence -> the decode step's residual rows, with statistics
__global__ void __launch_bounds__(256) gather_last(const float *x, int S, float *xd, float *stats, int d, int rms,
                                                   float eps) {
  __shared__ float scratch[4];
  const int b = blockIdx.x;
  const float *src = x + ((size_t)b * S + S - 1) * d;
  float *dst = xd + (size_t)b * d;
  for (int k = threadIdx.x; k < d; k += 256) dst[k] = src[k];
  __syncthreads();
  float mean, rstd;
  row_stats(dst, d, rms, eps, scratch, &mean, &rstd);
  if (threadIdx.x == 0) stats[b * 2] = mean, stats[b * 2 + 1] = rstd;
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

static void attn_plan(const Layout &L, int B, int max_rows, int *rows_per_block, int *splits) {
  // enough blocks to fill 256 CUs a few times over, at least 64 rows per block; the partial
  // buffer holds ceil(Smax/64) splits
  const int pairs = std::max(1, B * L.Hs);
  const int want = std::max(1, std::min(ceil_div(1024, pairs), L.attn_splits));
  int rpb = (int)align_up((size_t)ceil_div(L.Smax, want), 64);
  if (max_rows > 0 && rpb > max_rows) rpb = max_rows;
  *rows_per_block = rpb;
  *splits = ceil_div(L.Smax, rpb);
}

// ---------------------------------------------------------------------------
// the decode step as a list of phases
// ---------------------------------------------------------------------------
static float *xv(const Shard *g0, int v) { return (float *)(g0->ws + g0->L.ws_xv + (size_t)v * g0->L.xv_stride); }
static float *statv(const Shard *g0, int v) { return (float *)(g0->ws + g0->L.ws_statv) + (size_t)v * 64; }

static Phase lm_head_phase(Shard *const *group, int n_group, int B, const float *x, const float *stats, float *logits,
                           int32_t *next_tokens, int commit_inc, int target_blocks) {
  Shard *g0 = group[0];
  const Layout &L = g0->L;
  Phase ph = {};
  ph.kind = PH_LM_HEAD;
  SkinnyArgs &a = ph.g;
  a.w = g0->lm_head.ptr, a.tasks = g0->lm_head.row_tiles, a.k_blocks = g0->lm_head.k_blocks, a.B = B, a.N = L.V;
  plan_skinny(&a, L.esz, L.splitk_bytes, 1, target_blocks);
  a.x = x, a.stats = stats, a.gamma = g0->lnf_g, a.beta = g0->lnf_b;
  a.splitk = (float *)(g0->ws + L.ws_splitk), a.counters = (int *)(g0->ws + L.ws_counters);
  a.out_f32 = logits, a.ld_out = L.V;
  a.am_val = (float *)(g0->ws + L.ws_argmax);
  a.am_idx = (int *)(a.am_val + (size_t)ceil_div(a.tasks, 3) * 32);
  a.next_tokens = next_tokens;
  for (int i = 0; i < n_group; ++i) a.lens[i] = group[i]->d_len;
  a.n_lens = n_group, a.commit_inc = commit_inc;
  ph.gx = ceil_div(a.tasks, target_blocks < 0 ? 3 : 4), ph.gy = a.split;
  return ph;
}

// Phases of one decode step, in order.  Buffers follow the single-assignment rule: residual
// stream version v (0 = embedding, 2l+1 = after layer l's attention, 2l+2 = after its FFN), one
// q|k|v, attention-output and FFN-activation buffer per layer.
static void build_decode_plan(Shard *const *group, int n_group, const int32_t *tokens_in, int B, float *logits,
                              int32_t *next_tokens, int stop_after_layer, int target_blocks, std::vector<Phase> *plan) {
  Shard *g0 = group[0];
  const Layout &L0 = g0->L;
  const ss_model_desc &m = g0->m;
  const int dt = m.dtype, d = L0.d;
  const int FK = dt == SS_DTYPE_BF16 ? 32 : 16;
  const int rms = m.norm == SS_NORM_RMSNORM;
  float *stat_part = (float *)(g0->ws + L0.ws_stat_part);
  plan->clear();
  {
    Phase ph = {};
    ph.kind = PH_EMBED, ph.gx = B, ph.gy = 1;
    ph.e = EmbedArgs{tokens_in, g0->wte, g0->wpe, g0->d_len, 0, xv(g0, 0), statv(g0, 0), d, L0.V, rms, m.norm_eps};
    plan->push_back(ph);
  }
  // sum over the group at a reduce slot: shard i adds its partial to what the previous shards left
  auto resid = [&](int l, int i, const FragMat &w, const void *act, const float *bias, int v_in, int v_out) {
    Shard *s = group[i];
    const Layout &L = s->L;
    Phase ph = {};
    ph.kind = PH_RESID, ph.shard = i;
    SkinnyArgs &a = ph.g;
    a.w = w.ptr, a.tasks = w.row_tiles, a.k_blocks = w.k_blocks, a.B = B, a.N = d;
    plan_skinny(&a, L.esz, L.splitk_bytes, 1, target_blocks);
    a.act = act;
    a.splitk = (float *)(s->ws + L.ws_splitk), a.counters = (int *)(s->ws + L.ws_counters);
    a.bias = i == 0 ? bias : nullptr;
    const int pp0 = 2 * L0.Ls + 1;
    a.x_in = xv(g0, i == 0 ? v_in : pp0 + ((i - 1) & 1));
    a.x_resid = xv(g0, i == n_group - 1 ? v_out : pp0 + (i & 1));
    a.stat_part = stat_part, a.stats_out = statv(g0, v_out), a.rms = rms, a.eps = m.norm_eps;
    ph.gx = ceil_div(a.tasks, target_blocks < 0 ? 3 : 4), ph.gy = a.split;
    (void)l;
    plan->push_back(ph);
  };
  for (int l = 0; l < L0.Ls; ++l) {
    const LayerDev &D0 = g0->layers[l];
    for (int i = 0; i < n_group; ++i) {  // QKV projection of the new token
      Shard *s = group[i];
      const Layout &L = s->L;
      Phase ph = {};
      ph.kind = PH_QKV, ph.shard = i;
      SkinnyArgs &a = ph.g;
      a.w = s->wqkv[l].ptr, a.tasks = s->wqkv[l].row_tiles, a.k_blocks = s->wqkv[l].k_blocks, a.B = B, a.N = L.qkv_n;
      plan_skinny(&a, L.esz, L.splitk_bytes, 1, target_blocks);
      a.x = xv(g0, 2 * l), a.stats = statv(g0, 2 * l), a.gamma = D0.ln1_g, a.beta = D0.ln1_b;
      a.splitk = (float *)(s->ws + L.ws_splitk), a.counters = (int *)(s->ws + L.ws_counters);
      a.bias = s->layers[l].bqkv, a.out_f32 = (float *)(s->ws + L.ws_qkv_l + l * L.qkv_l_stride), a.ld_out = L.qkv_n;
      ph.gx = ceil_div(a.tasks, target_blocks < 0 ? 3 : 4), ph.gy = a.split;
      plan->push_back(ph);
    }
    for (int i = 0; i < n_group; ++i) {  // attention over the committed rows + append
      Shard *s = group[i];
      const Layout &L = s->L;
      Phase ph = {};
      ph.kind = PH_ATTN, ph.shard = i;
      DecodeAttnArgs &a = ph.at;
      a.qkv = (const float *)(s->ws + L.ws_qkv_l + l * L.qkv_l_stride);
      a.k_cache = s->kv_ptr(l, 0), a.v_cache = s->kv_ptr(l, 1);
      a.row_stride = s->kv_row_stride(), a.head_stride = s->kv_head_stride();
      a.lens = s->d_len, a.rope = m.pos == SS_POS_ROPE ? s->rope : nullptr;
      a.part = (float *)(s->ws + L.ws_attn_part);
      a.counters = (int *)(s->ws + L.ws_counters) + (L.n_counters - L.Bmax * L.Hs);
      a.o_out = s->ws + L.ws_o_l + l * L.o_l_stride;
      a.B = B, a.Hs = L.Hs, a.Dh = L.Dh, a.Smax = L.Smax, a.kv_dtype = s->m.kv_dtype;
      attn_plan(L, B, target_blocks < 0 ? 192 : 0, &a.rows_per_block, &a.splits);
      ph.gx = B * L.Hs, ph.gy = a.splits;
      plan->push_back(ph);
    }
    for (int i = 0; i < n_group; ++i)  // output projection, sum over the group, residual
      resid(l, i, group[i]->wo[l], group[i]->ws + group[i]->L.ws_o_l + l * group[i]->L.o_l_stride, D0.bo, 2 * l,
            2 * l + 1);
    for (int i = 0; i < n_group; ++i) {  // first FFN matrix + activation
      Shard *s = group[i];
      const Layout &L = s->L;
      const bool glu = m.act == SS_ACT_SWIGLU;
      Phase ph = {};
      ph.kind = PH_FFN_UP, ph.shard = i;
      SkinnyArgs &a = ph.g;
      a.w = s->w1[l].ptr, a.tasks = L.Fs / 16, a.k_blocks = s->w1[l].k_blocks, a.B = B, a.N = L.Fs;
      plan_skinny(&a, L.esz, L.splitk_bytes, glu ? 2 : 1, target_blocks);
      a.x = xv(g0, 2 * l + 1), a.stats = statv(g0, 2 * l + 1), a.gamma = D0.ln2_g, a.beta = D0.ln2_b;
      a.splitk = (float *)(s->ws + L.ws_splitk), a.counters = (int *)(s->ws + L.ws_counters);
      a.bias = s->layers[l].b1, a.act_out = s->ws + L.ws_u_l + l * L.u_l_stride, a.out_k_blocks = L.Fs / FK;
      a.act_kind = m.act;
      ph.gx = ceil_div(a.tasks, target_blocks < 0 ? 3 : 4), ph.gy = a.split;
      plan->push_back(ph);
    }
    for (int i = 0; i < n_group; ++i)  // second FFN matrix, sum over the group, residual
      resid(l, i, group[i]->w2[l], group[i]->ws + group[i]->L.ws_u_l + l * group[i]->L.u_l_stride, D0.b2, 2 * l + 1,
            2 * l + 2);
    if (l == stop_after_layer) return;
  }
  plan->push_back(lm_head_phase(group, n_group, B, xv(g0, 2 * L0.Ls), statv(g0, 2 * L0.Ls), logits, next_tokens, 1,
                                target_blocks));
}

// ---------------------------------------------------------------------------
// optional event bracket around one launch (measurement aid)
// ---------------------------------------------------------------------------
struct Bracket {
  Shard *sh;
  hipStream_t st;
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
  Bracket(Shard *s, int c, hipStream_t stream) : sh(s), st(stream), cls(c) {
    if (!sh->timing) return;
    e0 = get(sh), e1 = get(sh);
    if (e0) (void)hipEventRecord(e0, st);
  }
  ~Bracket() {
    if (!sh->timing || !e0 || !e1) return;
    (void)hipEventRecord(e1, st);
    sh->timed.push_back({cls, e0, e1});
  }
};

// one phase as a kernel of its own
static ss_status launch_phase(Shard *g0, const Phase &ph, hipStream_t st) {
  const int dt = g0->m.dtype;
  Bracket br(g0, ph.kind, st);
  switch (ph.kind) {
    case PH_EMBED:
      if (dt == SS_DTYPE_BF16) hipLaunchKernelGGL(embed_rows<bf16_t>, dim3(ph.gx), dim3(256), 0, st, ph.e);
      else hipLaunchKernelGGL(embed_rows<float>, dim3(ph.gx), dim3(256), 0, st, ph.e);
      SS_HIP(hipGetLastError());
      return SS_OK;
    case PH_QKV: return launch_skinny(dt, PRO_NORM, EPI_F32, ph.g, st);
    case PH_ATTN: return launch_decode_attn(dt, ph.at, st);
    case PH_RESID: return launch_skinny(dt, PRO_ACT, EPI_RESID, ph.g, st);
    case PH_FFN_UP: return launch_skinny(dt, PRO_NORM, g0->m.act == SS_ACT_SWIGLU ? EPI_SWIGLU : EPI_ACT, ph.g, st);
    case PH_LM_HEAD: return launch_skinny(dt, PRO_NORM, EPI_LOGITS, ph.g, st);
  }
  SS_FAIL(SS_EINVAL, "unknown phase kind %d", ph.kind);
}

static ss_status enqueue_decode(Shard *const *group, int n_group, const int32_t *tokens_in, int B, float *logits,
                                int32_t *next_tokens, hipStream_t st, int stop_after_layer) {
  std::vector<Phase> plan;
  build_decode_plan(group, n_group, tokens_in, B, logits, next_tokens, stop_after_layer, 0, &plan);
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

ss_status run_decode_step(Shard *const *group, int n_group, const int32_t *tokens_in, int B, float *logits,
                          int32_t *next_tokens, hipStream_t st, int stop_after_layer) {
  Shard *g0 = group[0];
  GraphKey key;
  key.B = B;
  key.ptrs = {tokens_in, logits, next_tokens, (const void *)st};
  for (int i = 0; i < n_group; ++i) key.ptrs.push_back(group[i]);
  const bool plain = !g0->timing && stop_after_layer < 0;
  static const int persistent_default = [] {
    // 0: graph / kernel-by-kernel (default); 1: persistent kernel; 2: wave-specialised persistent
    // kernel (switched off: a full-size run of it ended in a GPU fault whose cause is not yet known)
    const char *v = getenv("SS_PERSISTENT");
    return v && *v ? atoi(v) : 0;
  }();
  const int persistent_version = g0->persistent_mode >= 0 ? g0->persistent_mode : persistent_default;
  if (plain && n_group == 1 && persistent_version > 0) {
    const bool cached = g0->phases_valid && !(g0->phases_key < key) && !(key < g0->phases_key);
    std::vector<Phase> plan;
    const int blocks2 = persistent_version >= 2 ? persistent2_blocks(g0, B) : 0;
    if (blocks2 > 0) {
      if (!cached) build_decode_plan(group, n_group, tokens_in, B, logits, next_tokens, -1, -blocks2, &plan);
      return launch_persistent2_step(g0, plan, key, st);
    }
    if (persistent_supported(g0, B)) {
      if (!cached) build_decode_plan(group, n_group, tokens_in, B, logits, next_tokens, -1, 512, &plan);
      return launch_persistent_step(g0, plan, key, st);
    }
  }
  // the NULL stream cannot be captured, and a stream the caller is capturing is left to the caller
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  if (st) SS_HIP(hipStreamIsCapturing(st, &cs));
  const bool graph = g0->use_graph && plain && st != nullptr && cs == hipStreamCaptureStatusNone;
  if (!graph) return enqueue_decode(group, n_group, tokens_in, B, logits, next_tokens, st, stop_after_layer);
  auto it = g0->graphs.find(key);
  if (it == g0->graphs.end()) {
    hipGraph_t gr = nullptr;
    SS_HIP(hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
    ss_status rc = enqueue_decode(group, n_group, tokens_in, B, logits, next_tokens, st, -1);
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
    if (g0->graphs.size() >= 16) destroy_graphs(g0);
    it = g0->graphs.emplace(key, ex).first;
  }
  SS_HIP(hipGraphLaunch(it->second, st));
  return SS_OK;
}

// ---------------------------------------------------------------------------
// the initial phase
// ---------------------------------------------------------------------------
ss_status run_prefill(Shard *const *group, int n_group, const int32_t *tokens, int B, int S, float *logits,
                      int32_t *next_tokens, hipStream_t st) {
  Shard *g0 = group[0];
  const Layout &L0 = g0->L;
  const ss_model_desc &m = g0->m;
  const int dt = m.dtype, d = L0.d;
  const int FK = dt == SS_DTYPE_BF16 ? 32 : 16;
  const int rms = m.norm == SS_NORM_RMSNORM;
  const int T_live = B * S, T = (int)align_up((size_t)T_live, 128);
  const int parts = dt == SS_DTYPE_BF16 ? 2 : 1;  // bf16 GEMM inputs are hi/lo pairs
  for (int i = 0; i < n_group; ++i)
    if (T > group[i]->L.Tmax) SS_FAIL(SS_EINVAL, "%d prompt tokens exceed group[%d]'s workspace (%d)", T_live, i, group[i]->L.Tmax);
  float *x = (float *)(g0->ws + L0.ws_x);
  void *abuf = g0->ws + L0.ws_a;
  {
    EmbedArgs e{tokens, g0->wte, g0->wpe, nullptr, S, x, nullptr, d, L0.V, rms, m.norm_eps};
    if (dt == SS_DTYPE_BF16) hipLaunchKernelGGL(embed_rows<bf16_t>, dim3(T_live), dim3(256), 0, st, e);
    else hipLaunchKernelGGL(embed_rows<float>, dim3(T_live), dim3(256), 0, st, e);
    SS_HIP(hipGetLastError());
  }
  auto norm = [&](const float *g, const float *b) -> ss_status {
    if (dt == SS_DTYPE_BF16)
      hipLaunchKernelGGL(norm_rows<bf16_t>, dim3(T_live), dim3(256), 0, st, x, g, b, abuf, d, d / FK, rms, m.norm_eps);
    else
      hipLaunchKernelGGL(norm_rows<float>, dim3(T_live), dim3(256), 0, st, x, g, b, abuf, d, d / FK, rms, m.norm_eps);
    SS_HIP(hipGetLastError());
    return SS_OK;
  };
  for (int l = 0; l < L0.Ls; ++l) {
    const LayerDev &D0 = g0->layers[l];
    SS_TRY(norm(D0.ln1_g, D0.ln1_b));
    for (int i = 0; i < n_group; ++i) {
      Shard *s = group[i];
      const Layout &L = s->L;
      TileGemmArgs a = {};
      a.w = s->wqkv[l].ptr, a.row_tiles = s->wqkv[l].row_tiles, a.k_blocks = s->wqkv[l].k_blocks;
      a.act = abuf, a.act_parts = parts, a.T = T, a.T_live = T_live, a.N = L.qkv_n, a.bias = s->layers[l].bqkv;
      a.out_f32 = (float *)(s->ws + L.ws_qkv), a.ld_out = L.qkv_n;
      SS_TRY(launch_tile_gemm(dt, EPI_F32, a, st));
      PrefillAttnArgs p = {};
      p.qkv = (float *)(s->ws + L.ws_qkv);
      p.k_cache = s->kv_ptr(l, 0), p.v_cache = s->kv_ptr(l, 1);
      p.row_stride = s->kv_row_stride(), p.head_stride = s->kv_head_stride();
      p.rope = m.pos == SS_POS_ROPE ? s->rope : nullptr;
      p.o_out = s->ws + L.ws_o;
      p.B = B, p.S = S, p.Hs = L.Hs, p.Dh = L.Dh, p.Smax = L.Smax, p.kv_dtype = s->m.kv_dtype;
      SS_TRY(launch_prefill_kv_write(dt, p, st));
      SS_TRY(launch_prefill_attn(dt, p, st));
    }
    for (int i = 0; i < n_group; ++i) {
      Shard *s = group[i];
      const Layout &L = s->L;
      TileGemmArgs a = {};
      a.w = s->wo[l].ptr, a.row_tiles = s->wo[l].row_tiles, a.k_blocks = s->wo[l].k_blocks;
      a.act = s->ws + L.ws_o, a.act_parts = parts, a.T = T, a.T_live = T_live, a.N = d, a.bias = i == 0 ? D0.bo : nullptr;
      a.x_resid = x;
      SS_TRY(launch_tile_gemm(dt, EPI_RESID, a, st));
    }
    SS_TRY(norm(D0.ln2_g, D0.ln2_b));
    for (int i = 0; i < n_group; ++i) {
      Shard *s = group[i];
      const Layout &L = s->L;
      const bool glu = m.act == SS_ACT_SWIGLU;
      TileGemmArgs a = {};
      a.w = s->w1[l].ptr, a.row_tiles = s->w1[l].row_tiles, a.k_blocks = s->w1[l].k_blocks;
      a.act = abuf, a.act_parts = parts, a.T = T, a.T_live = T_live, a.N = L.Fs, a.bias = s->layers[l].b1;
      a.act_out = s->ws + L.ws_u, a.out_k_blocks = L.Fs / FK, a.out_parts = parts, a.act_kind = m.act;
      SS_TRY(launch_tile_gemm(dt, glu ? EPI_SWIGLU : EPI_ACT, a, st));
    }
    for (int i = 0; i < n_group; ++i) {
      Shard *s = group[i];
      const Layout &L = s->L;
      TileGemmArgs a = {};
      a.w = s->w2[l].ptr, a.row_tiles = s->w2[l].row_tiles, a.k_blocks = s->w2[l].k_blocks;
      a.act = s->ws + L.ws_u, a.act_parts = parts, a.T = T, a.T_live = T_live, a.N = d, a.bias = i == 0 ? D0.b2 : nullptr;
      a.x_resid = x;
      SS_TRY(launch_tile_gemm(dt, EPI_RESID, a, st));
    }
  }
  float *xd = xv(g0, 2 * L0.Ls);
  float *stats = statv(g0, 2 * L0.Ls);
  hipLaunchKernelGGL(gather_last, dim3(B), dim3(256), 0, st, x, S, xd, stats, d, rms, m.norm_eps);
  SS_HIP(hipGetLastError());
  const Phase ph = lm_head_phase(group, n_group, B, xd, stats, logits, next_tokens, S, 0);
  return launch_skinny(dt, PRO_NORM, EPI_LOGITS, ph.g, st);
}

}  // namespace ss

using namespace ss;

extern "C" {

ss_status ss_prefill(ss_shard *const *group_, int32_t n_group, const int32_t *tokens, int32_t B, int32_t S_in,
                     float *logits, int32_t *next_tokens, void *hip_stream) {
  Shard *const *group = (Shard *const *)group_;
  if (!tokens) SS_FAIL(SS_EINVAL, "tokens is NULL");
  SS_TRY(check_group(group, n_group, B));
  if (S_in < 1) SS_FAIL(SS_EINVAL, "S_in must be positive");
  for (int i = 0; i < n_group; ++i) {
    if (S_in > group[i]->L.Smax) SS_FAIL(SS_EINVAL, "S_in %d exceeds group[%d]'s max_seq %d", S_in, i, group[i]->L.Smax);
    for (int b = 0; b < B; ++b)
      if (group[i]->h_len[b] != 0) SS_FAIL(SS_ESTATE, "row %d of group[%d] already holds %d tokens", b, i, group[i]->h_len[b]);
  }
  SS_TRY(run_prefill(group, n_group, tokens, B, S_in, logits, next_tokens, (hipStream_t)hip_stream));
  for (int i = 0; i < n_group; ++i)
    for (int b = 0; b < B; ++b) group[i]->h_len[b] = S_in;
  return SS_OK;
}

// Host-only check aid: the phase table of one decode step for a shard of the given shape whose
// device memory starts at address `fake_base` (nothing is allocated or launched).  Writes up to
// max_phases Phase records to out_phases, the layout's total bytes to out_total, returns the
// number of phases (negative on error).  mode: 0 kernel-by-kernel plan, > 0 resident blocks of
// the persistent kernel (1: block bodies, 2: wave-specialised).
int32_t ss_debug_plan(const ss_model_desc *desc, const ss_slice *slice, int32_t max_batch, int32_t max_seq, int32_t B,
                      int32_t mode, int32_t blocks, uint64_t fake_base, void *out_phases, int32_t max_phases,
                      uint64_t *out_total, uint64_t *out_sizeof_phase) {
  if (!desc || !slice || validate_desc(*desc, *slice, max_batch, max_seq) != SS_OK) return -1;
  Shard sh;
  sh.m = *desc, sh.s = *slice;
  compute_layout(*desc, *slice, max_batch, max_seq, &sh.L);
  const Layout &L = sh.L;
  sh.base = (char *)fake_base;
  sh.wte = sh.base + L.off_wte, sh.wpe = L.max_pos ? sh.base + L.off_wpe : nullptr;
  sh.lnf_g = (float *)(sh.base + L.off_lnf_g), sh.lnf_b = (float *)(sh.base + L.off_lnf_b);
  sh.rope = (float2 *)(sh.base + L.off_rope), sh.kv = sh.base + L.off_kv, sh.d_len = (int32_t *)(sh.base + L.off_len);
  sh.ws = sh.base + L.off_ws;
  const int FK = desc->dtype == SS_DTYPE_BF16 ? 32 : 16, d = L.d, HD = L.Hs * L.Dh;
  sh.lm_head = FragMat{sh.base + L.off_lm, L.V, d, ceil_div(L.V, 16), d / FK};
  sh.layers.resize(L.Ls), sh.wqkv.resize(L.Ls), sh.wo.resize(L.Ls), sh.w1.resize(L.Ls), sh.w2.resize(L.Ls);
  for (int l = 0; l < L.Ls; ++l) {
    char *lb = sh.base + L.off_layer[l];
    sh.wqkv[l] = FragMat{lb + L.lo_wqkv, L.qkv_n, d, L.qkv_n / 16, d / FK};
    sh.wo[l] = FragMat{lb + L.lo_wo, d, HD, d / 16, HD / FK};
    sh.w1[l] = FragMat{lb + L.lo_w1, L.w1_rows, d, L.w1_rows / 16, d / FK};
    sh.w2[l] = FragMat{lb + L.lo_w2, d, L.Fs, d / 16, L.Fs / FK};
    LayerDev &D = sh.layers[l];
    D.ln1_g = (float *)(lb + L.lo_ln1_g), D.ln1_b = (float *)(lb + L.lo_ln1_b);
    D.ln2_g = (float *)(lb + L.lo_ln2_g), D.ln2_b = (float *)(lb + L.lo_ln2_b);
    D.bqkv = (float *)(lb + L.lo_bqkv), D.bo = (float *)(lb + L.lo_bo), D.b1 = (float *)(lb + L.lo_b1),
    D.b2 = (float *)(lb + L.lo_b2);
  }
  Shard *group[1] = {&sh};
  std::vector<Phase> plan;
  build_decode_plan(group, 1, (const int32_t *)8, B, (float *)16, (int32_t *)24, -1, mode == 0 ? 0 : (mode == 1 ? blocks : -blocks),
                    &plan);
  if (out_total) *out_total = L.total;
  if (out_sizeof_phase) *out_sizeof_phase = sizeof(Phase);
  const int n = (int)plan.size();
  if (out_phases)
    for (int i = 0; i < n && i < max_phases; ++i) memcpy((char *)out_phases + (size_t)i * sizeof(Phase), &plan[i], sizeof(Phase));
  return n;
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

ss_status ss_decode_step(ss_shard *const *group_, int32_t n_group, const int32_t *tokens_in, int32_t B, float *logits,
                         int32_t *next_tokens, void *hip_stream) {
  Shard *const *group = (Shard *const *)group_;
  if (!tokens_in) SS_FAIL(SS_EINVAL, "tokens_in is NULL");
  SS_TRY(check_group(group, n_group, B));
  for (int b = 0; b < B; ++b) {
    const int n = group[0]->h_len[b];
    for (int i = 0; i < n_group; ++i) {
      if (group[i]->h_len[b] != n)
        SS_FAIL(SS_ESTATE, "row %d: group[%d] committed %d tokens, group[0] %d", b, i, group[i]->h_len[b], n);
      if (n + 1 > group[i]->L.Smax) SS_FAIL(SS_ESTATE, "row %d: cache of group[%d] is full (%d rows)", b, i, n);
    }
  }
  int stop = -1;
  for (int i = 0; i < n_group; ++i) stop = std::max(stop, group[i]->interrupt_after);
  ss_status rc = run_decode_step(group, n_group, tokens_in, B, logits, next_tokens, (hipStream_t)hip_stream, stop);
  if (rc != SS_OK) return rc;  // SS_EINTR: nothing committed
  for (int i = 0; i < n_group; ++i)
    for (int b = 0; b < B; ++b) group[i]->h_len[b] += 1;
  return SS_OK;
}

}  // extern "C"
