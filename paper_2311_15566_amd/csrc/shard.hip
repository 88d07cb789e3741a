// Shard object: device-memory carve-up, model-context upload into matrix-core operand
// order, cache-context export/import and the KV head re-partition kernel.
#include "shard.h"

#include <math.h>
#include <stdarg.h>
#include <string.h>

#include <algorithm>
#include <new>

namespace ss {

// ---------------------------------------------------------------------------
// errors
// ---------------------------------------------------------------------------
static thread_local char g_err[512] = "";
void set_error(const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

// ---------------------------------------------------------------------------
// validation + layout
// ---------------------------------------------------------------------------
ss_status validate_desc(const ss_model_desc &m, const ss_slice &s, int max_batch, int max_seq) {
  if (m.n_layers <= 0 || m.d_model <= 0 || m.n_heads <= 0 || m.ffn <= 0 || m.vocab <= 0)
    SS_FAIL(SS_EINVAL, "model descriptor has a non-positive dimension");
  if (m.head_dim != 64 && m.head_dim != 128) SS_FAIL(SS_EINVAL, "head_dim must be 64 or 128 (got %d)", m.head_dim);
  if (m.d_model % 64 || m.d_model > 16384)
    SS_FAIL(SS_EINVAL, "d_model must be a multiple of 64, at most 16384 (got %d)", m.d_model);
  if (m.dtype != SS_DTYPE_F32 && m.dtype != SS_DTYPE_BF16) SS_FAIL(SS_EINVAL, "unknown dtype %d", m.dtype);
  if (m.dtype == SS_DTYPE_F32 ? m.kv_dtype != SS_DTYPE_F32 : (m.kv_dtype != SS_DTYPE_F16 && m.kv_dtype != SS_DTYPE_BF16))
    SS_FAIL(SS_EINVAL, "kv_dtype %d does not go with dtype %d", m.kv_dtype, m.dtype);
  if (m.norm != SS_NORM_LAYERNORM && m.norm != SS_NORM_RMSNORM) SS_FAIL(SS_EINVAL, "unknown norm %d", m.norm);
  if (m.act < SS_ACT_GELU_TANH || m.act > SS_ACT_SWIGLU) SS_FAIL(SS_EINVAL, "unknown activation %d", m.act);
  if (m.pos != SS_POS_LEARNED && m.pos != SS_POS_ROPE) SS_FAIL(SS_EINVAL, "unknown position scheme %d", m.pos);
  if (!(0 <= s.layer_lo && s.layer_lo < s.layer_hi && s.layer_hi <= m.n_layers))
    SS_FAIL(SS_EINVAL, "layer interval [%d,%d) not inside [0,%d)", s.layer_lo, s.layer_hi, m.n_layers);
  if (!(0 <= s.head_lo && s.head_lo < s.head_hi && s.head_hi <= m.n_heads))
    SS_FAIL(SS_EINVAL, "head interval [%d,%d) not inside [0,%d)", s.head_lo, s.head_hi, m.n_heads);
  if (!(0 <= s.ffn_lo && s.ffn_lo < s.ffn_hi && s.ffn_hi <= m.ffn))
    SS_FAIL(SS_EINVAL, "FFN interval [%d,%d) not inside [0,%d)", s.ffn_lo, s.ffn_hi, m.ffn);
  if ((s.ffn_hi - s.ffn_lo) % 64) SS_FAIL(SS_EINVAL, "FFN slice width must be a multiple of 64");
  if (max_batch < 1 || max_batch > 32) SS_FAIL(SS_EINVAL, "max_batch must be in [1,32] (got %d)", max_batch);
  if (max_seq < 1 || max_seq > 65536) SS_FAIL(SS_EINVAL, "max_seq must be in [1,65536] (got %d)", max_seq);
  if (m.pos == SS_POS_LEARNED && m.max_pos < max_seq)
    SS_FAIL(SS_EINVAL, "learned position table (%d rows) shorter than max_seq %d", m.max_pos, max_seq);
  return SS_OK;
}

static size_t frag_bytes(int rows, int K, int esz) {
  int fk = esz == 2 ? 32 : 16;
  return (size_t)ceil_div(rows, 16) * ceil_div(K, fk) * 1024;
}

bool compute_layout(const ss_model_desc &m, const ss_slice &s, int max_batch, int max_seq, Layout *L) {
  L->Ls = s.layer_hi - s.layer_lo;
  L->Hs = s.head_hi - s.head_lo;
  L->Fs = s.ffn_hi - s.ffn_lo;
  L->d = m.d_model;
  L->Dh = m.head_dim;
  L->V = m.vocab;
  L->max_pos = m.pos == SS_POS_LEARNED ? m.max_pos : 0;
  L->Bmax = max_batch;
  L->Smax = max_seq;
  L->esz = m.dtype == SS_DTYPE_BF16 ? 2 : 4;
  L->Bpad = (int)align_up(max_batch, 16);
  L->Tmax = (int)align_up((size_t)max_batch * max_seq, 256);
  L->qkv_n = 3 * L->Hs * L->Dh;
  L->w1_rows = m.act == SS_ACT_SWIGLU ? 2 * L->Fs : L->Fs;
  L->attn_splits = ceil_div(max_seq, 64);
  const int esz = L->esz, d = L->d, HD = L->Hs * L->Dh;
  size_t o = 0;
  auto take = [&](size_t bytes) {
    size_t at = o;
    o = align_up(o + bytes, 256);
    return at;
  };
  L->off_wte = take((size_t)L->V * d * esz);
  L->off_wpe = take((size_t)L->max_pos * d * esz);
  L->off_lm = take(frag_bytes(L->V, d, esz));
  L->off_lnf_g = take((size_t)d * 4);
  L->off_lnf_b = take((size_t)d * 4);
  L->off_wg_lm = take(align_up((size_t)L->V, 16) * 4);
  L->off_cb_lm = take(align_up((size_t)L->V, 16) * 4);
  L->off_rope = take((size_t)max_seq * (L->Dh / 2) * sizeof(float2));
  // one layer's block
  size_t lo = 0;
  auto ltake = [&](size_t bytes) {
    size_t at = lo;
    lo = align_up(lo + bytes, 256);
    return at;
  };
  L->lo_ln1_g = ltake((size_t)d * 4);
  L->lo_ln1_b = ltake((size_t)d * 4);
  L->lo_ln2_g = ltake((size_t)d * 4);
  L->lo_ln2_b = ltake((size_t)d * 4);
  L->lo_wqkv = ltake(frag_bytes(L->qkv_n, d, esz));
  L->lo_bqkv = ltake((size_t)L->qkv_n * 4);
  L->lo_wo = ltake(frag_bytes(d, HD, esz));
  L->lo_bo = ltake((size_t)d * 4);
  L->lo_w1 = ltake(frag_bytes(L->w1_rows, d, esz));
  L->lo_b1 = ltake((size_t)L->w1_rows * 4);
  L->lo_w2 = ltake(frag_bytes(d, L->Fs, esz));
  L->lo_b2 = ltake((size_t)d * 4);
  L->lo_wg_qkv = ltake((size_t)L->qkv_n * 4);
  L->lo_cb_qkv = ltake((size_t)L->qkv_n * 4);
  L->lo_wg_1 = ltake((size_t)L->w1_rows * 4);
  L->lo_cb_1 = ltake((size_t)L->w1_rows * 4);
  L->layer_bytes = lo;
  L->off_layer.clear();
  for (int l = 0; l < L->Ls; ++l) L->off_layer.push_back(take(L->layer_bytes));
  L->kv_bytes = (size_t)L->Ls * 2 * max_batch * L->Hs * max_seq * L->Dh * esz;
  L->off_kv = take(L->kv_bytes);
  L->off_len = take((size_t)32 * 4);
  L->off_zero = take((size_t)1024);
  // workspace
  size_t w = 0;
  auto wtake = [&](size_t bytes) {
    size_t at = w;
    w = align_up(w + bytes, 256);
    return at;
  };
  const int T = L->Tmax;
  L->ws_x = wtake((size_t)T * d * 4);
  L->ws_a = wtake((size_t)T * d * esz);  // operands of the initial phase: halves (bf16 models) or floats
  // Models with rotary positions: their attention scores are several times more sensitive to the rounding of
  // the normalised input to 11 bits than the others', and the prompt's keys carry that error into every later
  // step, so the initial phase computes q and k from a two-part operand (22 bits).
  L->two_part_qk = m.pos == SS_POS_ROPE && m.dtype == SS_DTYPE_BF16;
  L->ws_a_lo = wtake(L->two_part_qk ? (size_t)T * d * esz : 0);
  L->ws_qkv = wtake((size_t)T * L->qkv_n * 4);
  L->ws_o = wtake((size_t)T * HD * esz);
  L->ws_u = wtake((size_t)T * L->Fs * esz);
  L->ws_vt = wtake((size_t)max_batch * L->Hs * L->Dh * align_up((size_t)max_seq, 64) * 2);
  L->ws_pstat = wtake((size_t)(2 * ceil_div(d, 128) + 2) * T * 8);  // partial sums, then (mean, rstd, mean - centre, -) per token
  {
    const int fk = esz == 2 ? 32 : 16;  // one 1 KiB operand fragment per 16 rows and k block
    L->ws_xd = wtake((size_t)32 * d * 4);
    L->ws_ad = wtake((size_t)2 * (d / fk) * 1024);
    L->ws_statd = wtake((size_t)(d / 32) * 32 * 4 * 4);
    L->ws_cen = wtake((size_t)32 * 4);
    L->ws_qkvd = wtake((size_t)kQkvParts * 32 * L->qkv_n * 4);  // partial sums when the GEMM cuts K into slices
    L->ws_od = wtake((size_t)2 * (HD / fk) * 1024);
    L->ws_ud = wtake((size_t)2 * (L->Fs / fk) * 1024);
  }
  L->n_counters = 16 + max_batch * L->Hs;  // [16..): decode attention's arrival counters, per (row, head); [0..16) unused
  L->ws_counters = wtake((size_t)L->n_counters * 4);
  L->ws_attn_part = wtake((size_t)max_batch * L->Hs * L->attn_splits * (L->Dh + 4) * 4);
  L->ws_argmax = wtake((size_t)ceil_div(L->V, 16) * 32 * 8);  // per LM-head block and row a best logit and its index; at most a block per weight tile
  L->ffnpart_bytes = (max_batch > 16 && m.act != SS_ACT_SWIGLU) ? (size_t)kQkvParts * 32 * L->Fs * 4 : 0;
  L->ws_ffnpart = wtake(L->ffnpart_bytes);
  L->ws_dec_end = w;
  // upload staging shares the workspace: it must hold the largest raw tensor slice
  size_t stage = std::max((size_t)L->V * d, (size_t)d * std::max(std::max(HD, L->Fs), 1)) * esz;
  L->ws_bytes = std::max(w, align_up(stage, 256));
  L->off_ws = take(L->ws_bytes);
  L->total = o;
  return true;
}

// ---------------------------------------------------------------------------
// kernels used at creation
// ---------------------------------------------------------------------------
// src: raw slice; element (n, k) at src[n*sn + k*sk].  dst: fragments; logical row tile t of
// the slice lands at tile t*tile_mul + tile_add (SwiGLU gate/up interleave).  Rows >= N and
// k >= K are zero-filled.  The fragments hold the GEMM operand type (bf16 weights become halves).
template <typename T>
__global__ void __launch_bounds__(256) shuffle_to_frags(const T *__restrict__ src, T *__restrict__ dst, int N, int K,
                                                        size_t sn, size_t sk, int k_blocks, int tile_mul,
                                                        int tile_add, int row_tiles) {
  constexpr int PL = Elem<T>::kPerLane, FK = Elem<T>::kFragK;
  size_t total = (size_t)row_tiles * k_blocks * 64;  // one thread per 16-byte lane piece
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    int lane = (int)(i & 63);
    size_t frag = i >> 6;
    int kb = (int)(frag % k_blocks);
    int t = (int)(frag / k_blocks);
    int n = t * 16 + (lane & 15);
    int k0 = kb * FK + (lane >> 4) * PL;
    T v[PL];
#pragma unroll
    for (int j = 0; j < PL; ++j) {
      int k = k0 + j;
      v[j] = (n < N && k < K) ? src[(size_t)n * sn + (size_t)k * sk] : (T)0;
    }
    typedef typename Operand<T>::type WT;
    static_assert(sizeof(WT) == sizeof(T), "operand and weight elements have one size");
    WT *o = (WT *)dst + ((size_t)(t * tile_mul + tile_add) * k_blocks + kb) * (64 * PL) + lane * PL;
#pragma unroll
    for (int j = 0; j < PL; ++j) o[j] = Elem<WT>::from_f32(Elem<T>::to_f32(v[j]));
  }
}

__global__ void fill_i32(int32_t *p, int n, int32_t v) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// ---------------------------------------------------------------------------
// KV head re-partition: a pure move.  Segment = (layer, K|V, mapped row, head): n rows of
// Dh elements, contiguous in both layouts.  One block copies one 4 KiB piece of one segment with
// 16-byte accesses; lengths come from the host mirror (blocks past a shorter row's end exit at once).
// ---------------------------------------------------------------------------
struct RepackArgs {
  const char *src;
  char *dst;
  size_t s_layer, s_plane, s_row, s_head;  // source strides in bytes
  size_t d_layer, d_plane, d_row, d_head;  // destination strides in bytes
  int n_layers, n_heads;                   // intersection extents
  int row_bytes;                           // Dh * esz
  int n_map;                               // mapped destination rows
  int chunks_per_seg;                      // grid.x: blocks per segment of the longest mapped row
  int chunk_vec;                           // 16-byte vectors per block
  int32_t map_dst[32], map_src[32], map_len[32];
  int32_t *dst_len;                        // device lengths of dst
};

// the destination's lengths are set after the rows have landed (stream order)
__global__ void kv_repack_commit(RepackArgs a) {
  if (threadIdx.x < a.n_map) a.dst_len[a.map_dst[threadIdx.x]] = a.map_len[threadIdx.x];
}

// grid = (4 KiB pieces of the longest segment, mapped rows x heads, layers x {K, V}); a thread moves one
// 16-byte vector.  Many small blocks, one access per lane: measured on this chip, a copy laid out this way moves
// 6.4-6.6 TB/s (read + written) where blocks of 64 KiB with four loads in flight per lane move 5.6 and the
// runtime's own device-to-device copy 5.0.
__global__ void __launch_bounds__(256) kv_repack_kernel(RepackArgs a) {
  const int r = blockIdx.y / a.n_heads, h = blockIdx.y - r * a.n_heads;
  const int l = blockIdx.z >> 1, c = blockIdx.z & 1;
  const size_t nvec = ((size_t)a.map_len[r] * a.row_bytes) >> 4;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= nvec) return;
  const u32x4 *s = (const u32x4 *)(a.src + l * a.s_layer + c * a.s_plane + a.map_src[r] * a.s_row + h * a.s_head);
  u32x4 *d = (u32x4 *)(a.dst + l * a.d_layer + c * a.d_plane + a.map_dst[r] * a.d_row + h * a.d_head);
  __builtin_nontemporal_store(__builtin_nontemporal_load(s + i), d + i);
}

// ---------------------------------------------------------------------------
// Model-context re-slice: batched strided copies between resident shards.  A descriptor is
// `rows` runs of `row_bytes` (a multiple of 16) with their own strides in source and
// destination; block b finds its descriptor by bisection over the descriptors' first blocks and
// copies up to 16 KiB of it with 16-byte accesses.
// ---------------------------------------------------------------------------
struct Copy2D {
  const char *src;
  char *dst;
  uint64_t src_stride, dst_stride;
  uint32_t rows, row_bytes;
  uint32_t rows_per_block;  // >= 1; when 1, a row may take several blocks of chunk_vec vectors
  uint32_t blocks_per_row;  // >= 1
  uint32_t first_block;
  uint32_t pad;
};

__global__ void __launch_bounds__(256) copy2d_kernel(const Copy2D *__restrict__ desc, int n_desc) {
  int lo = 0, hi = n_desc - 1;
  while (lo < hi) {  // last descriptor whose first block is <= blockIdx.x
    const int mid = (lo + hi + 1) >> 1;
    if (desc[mid].first_block <= blockIdx.x) lo = mid;
    else hi = mid - 1;
  }
  const Copy2D c = desc[lo];
  const uint32_t local = blockIdx.x - c.first_block;
  const uint32_t row_vec = c.row_bytes >> 4;
  if (c.rows_per_block > 1) {
    const uint32_t r0 = local * c.rows_per_block, r1 = min(c.rows, r0 + c.rows_per_block);
    const uint32_t total = (r1 - r0) * row_vec;
    for (uint32_t i = threadIdx.x; i < total; i += 256) {
      const uint32_t r = r0 + i / row_vec, v = i % row_vec;
      const u32x4 x = __builtin_nontemporal_load((const u32x4 *)(c.src + (size_t)r * c.src_stride) + v);
      __builtin_nontemporal_store(x, (u32x4 *)(c.dst + (size_t)r * c.dst_stride) + v);
    }
  } else {
    const uint32_t r = local / c.blocks_per_row, part = local % c.blocks_per_row;
    const uint32_t v0 = part * 1024u, v1 = min(row_vec, v0 + 1024u);
    const u32x4 *sp = (const u32x4 *)(c.src + (size_t)r * c.src_stride);
    u32x4 *dp = (u32x4 *)(c.dst + (size_t)r * c.dst_stride);
    uint32_t i = v0 + threadIdx.x;
    for (; i + 768 < v1; i += 1024) {
      const u32x4 x0 = __builtin_nontemporal_load(sp + i), x1 = __builtin_nontemporal_load(sp + i + 256);
      const u32x4 x2 = __builtin_nontemporal_load(sp + i + 512), x3 = __builtin_nontemporal_load(sp + i + 768);
      __builtin_nontemporal_store(x0, dp + i);
      __builtin_nontemporal_store(x1, dp + i + 256);
      __builtin_nontemporal_store(x2, dp + i + 512);
      __builtin_nontemporal_store(x3, dp + i + 768);
    }
    for (; i < v1; i += 256) __builtin_nontemporal_store(__builtin_nontemporal_load(sp + i), dp + i);
  }
}

}  // namespace ss

using namespace ss;

// ---------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------
extern "C" {

const char *ss_last_error(void) { return g_err; }
const char *ss_version(void) { return "spotshard 0.1 (gfx950)"; }

size_t ss_shard_device_bytes(const ss_model_desc *desc, const ss_slice *slice, int32_t max_batch, int32_t max_seq) {
  if (!desc || !slice) return 0;
  if (validate_desc(*desc, *slice, max_batch, max_seq) != SS_OK) return 0;
  Layout L;
  compute_layout(*desc, *slice, max_batch, max_seq, &L);
  return L.total;
}

}  // extern "C"

namespace ss {

void bind_pointers(Shard *sh) {
  const Layout &L = sh->L;
  const ss_model_desc &m = sh->m;
  const int FK = m.dtype == SS_DTYPE_BF16 ? 32 : 16, d = L.d, HD = L.Hs * L.Dh;
  const bool bias = m.has_bias, ln = m.norm == SS_NORM_LAYERNORM, glu = m.act == SS_ACT_SWIGLU;
  char *base = sh->base;
  sh->wte = base + L.off_wte;
  sh->wpe = L.max_pos ? base + L.off_wpe : nullptr;
  sh->lnf_g = (float *)(base + L.off_lnf_g);
  sh->lnf_b = ln ? (float *)(base + L.off_lnf_b) : nullptr;
  sh->wg_lm = ln ? (float *)(base + L.off_wg_lm) : nullptr;
  sh->cb_lm = ln ? (float *)(base + L.off_cb_lm) : nullptr;
  sh->rope = (float2 *)(base + L.off_rope);
  sh->kv = base + L.off_kv;
  sh->d_len = (int32_t *)(base + L.off_len);
  sh->zero_frag = base + L.off_zero;
  sh->ws = base + L.off_ws;
  sh->dec = sh->ws + L.ws_xd;
  sh->lm_head = FragMat{base + L.off_lm, L.V, d, ceil_div(L.V, 16), d / FK};
  sh->layers.resize(L.Ls);
  sh->wqkv.resize(L.Ls), sh->wo.resize(L.Ls), sh->w1.resize(L.Ls), sh->w2.resize(L.Ls);
  sh->wg_qkv.resize(L.Ls), sh->cb_qkv.resize(L.Ls), sh->wg_1.resize(L.Ls), sh->cb_1.resize(L.Ls);
  for (int l = 0; l < L.Ls; ++l) {
    char *lb = base + L.off_layer[l];
    sh->wqkv[l] = FragMat{lb + L.lo_wqkv, L.qkv_n, d, L.qkv_n / 16, d / FK};
    sh->wo[l] = FragMat{lb + L.lo_wo, d, HD, d / 16, HD / FK};
    sh->w1[l] = FragMat{lb + L.lo_w1, L.w1_rows, d, L.w1_rows / 16, d / FK};
    sh->w2[l] = FragMat{lb + L.lo_w2, d, L.Fs, d / 16, L.Fs / FK};
    LayerDev &D = sh->layers[l];
    D.ln1_g = (float *)(lb + L.lo_ln1_g), D.ln1_b = ln ? (float *)(lb + L.lo_ln1_b) : nullptr;
    D.ln2_g = (float *)(lb + L.lo_ln2_g), D.ln2_b = ln ? (float *)(lb + L.lo_ln2_b) : nullptr;
    D.wqkv = sh->wqkv[l].ptr, D.bqkv = bias ? (float *)(lb + L.lo_bqkv) : nullptr;
    D.wo = sh->wo[l].ptr, D.bo = bias ? (float *)(lb + L.lo_bo) : nullptr;
    D.w1 = sh->w1[l].ptr, D.b1 = (bias && !glu) ? (float *)(lb + L.lo_b1) : nullptr;
    D.w2 = sh->w2[l].ptr, D.b2 = bias ? (float *)(lb + L.lo_b2) : nullptr;
    // LayerNorm folds gamma and beta (+ bias); RMSNorm needs neither, a bias alone stays a bias
    sh->wg_qkv[l] = ln ? (float *)(lb + L.lo_wg_qkv) : nullptr;
    sh->cb_qkv[l] = ln ? (float *)(lb + L.lo_cb_qkv) : const_cast<float *>(D.bqkv);
    sh->wg_1[l] = ln ? (float *)(lb + L.lo_wg_1) : nullptr;
    sh->cb_1[l] = ln ? (float *)(lb + L.lo_cb_1) : const_cast<float *>(D.b1);
  }
}

template <typename T>
static ss_status upload_matrix(Shard *sh, hipStream_t st, const void *host, size_t host_ld, size_t row0, size_t col0,
                               size_t rows, size_t cols, bool rows_are_out, void *dst, int k_blocks, int row_tiles,
                               int tile_mul, int tile_add) {
  // host: row-major [*, host_ld]; take rows [row0,row0+rows) x cols [col0,col0+cols) into staging (dense)
  if (!host) SS_FAIL(SS_EINVAL, "a required weight pointer is NULL");
  T *stage = (T *)sh->ws;
  const T *h = (const T *)host + row0 * host_ld + col0;
  if (cols == host_ld)
    SS_HIP(hipMemcpyAsync(stage, h, rows * cols * sizeof(T), hipMemcpyHostToDevice, st));
  else
    SS_HIP(hipMemcpy2DAsync(stage, cols * sizeof(T), h, host_ld * sizeof(T), cols * sizeof(T), rows,
                            hipMemcpyHostToDevice, st));
  int N, K;
  size_t sn, sk;
  if (rows_are_out) {  // staging is [N][K]
    N = (int)rows, K = (int)cols, sn = cols, sk = 1;
  } else {             // staging is [K][N]
    N = (int)cols, K = (int)rows, sn = 1, sk = cols;
  }
  size_t total = (size_t)row_tiles * k_blocks * 64;
  int blocks = (int)std::min<size_t>((total + 255) / 256, 65535);
  hipLaunchKernelGGL(shuffle_to_frags<T>, dim3(blocks), dim3(256), 0, st, stage, (T *)dst, N, K, sn, sk, k_blocks,
                     tile_mul, tile_add, row_tiles);
  SS_HIP(hipGetLastError());
  return SS_OK;
}

static ss_status upload_vec(hipStream_t st, const void *host, size_t off, size_t n, float *dst, bool required) {
  if (!host) {
    if (required) SS_FAIL(SS_EINVAL, "a required vector pointer is NULL");
    return SS_OK;
  }
  SS_HIP(hipMemcpyAsync(dst, (const float *)host + off, n * 4, hipMemcpyHostToDevice, st));
  return SS_OK;
}

template <typename T>
static ss_status upload_all(Shard *sh, const ss_weights *P, hipStream_t st) {
  const Layout &L = sh->L;
  const ss_model_desc &m = sh->m;
  const int d = L.d, Dh = L.Dh, HD = L.Hs * Dh;
  const int FK = Elem<T>::kFragK;
  const int Hp = P->slice.head_hi - P->slice.head_lo, Fp = P->slice.ffn_hi - P->slice.ffn_lo;
  const size_t c0 = (size_t)(sh->s.head_lo - P->slice.head_lo) * Dh;  // column offset of our heads in the parent
  const size_t f0 = (size_t)(sh->s.ffn_lo - P->slice.ffn_lo);
  const bool bias = m.has_bias, ln = m.norm == SS_NORM_LAYERNORM;
  if (!P->wte || !P->lm_head || !P->lnf_g) SS_FAIL(SS_EINVAL, "wte / lm_head / lnf_g must not be NULL");
  SS_HIP(hipMemcpyAsync(sh->wte, P->wte, (size_t)L.V * d * sizeof(T), hipMemcpyHostToDevice, st));
  if (m.pos == SS_POS_LEARNED) {
    if (!P->wpe) SS_FAIL(SS_EINVAL, "wpe is NULL for a learned-position model");
    SS_HIP(hipMemcpyAsync(sh->wpe, P->wpe, (size_t)L.max_pos * d * sizeof(T), hipMemcpyHostToDevice, st));
  }
  SS_TRY(upload_matrix<T>(sh, st, P->lm_head, d, 0, 0, L.V, d, true, sh->lm_head.ptr, d / FK, ceil_div(L.V, 16), 1, 0));
  SS_TRY(upload_vec(st, P->lnf_g, 0, d, sh->lnf_g, true));
  SS_TRY(upload_vec(st, P->lnf_b, 0, d, sh->lnf_b, ln));
  if (ln)
    SS_TRY(launch_fold_norm(m.dtype, sh->lm_head.ptr, sh->lm_head.row_tiles, sh->lm_head.k_blocks, sh->lnf_g, sh->lnf_b,
                            nullptr, sh->wg_lm, sh->cb_lm, st));
  for (int l = 0; l < L.Ls; ++l) {
    const ss_layer_weights &W = P->layers[sh->s.layer_lo - P->slice.layer_lo + l];
    char *lb = sh->base + L.off_layer[l];
    const LayerDev &D = sh->layers[l];
    // the vectors are uploaded to their slots whether or not the model uses them
    float *bqkv = (float *)(lb + L.lo_bqkv), *bo = (float *)(lb + L.lo_bo), *b1 = (float *)(lb + L.lo_b1),
          *b2 = (float *)(lb + L.lo_b2);
    SS_TRY(upload_vec(st, W.ln1_g, 0, d, (float *)(lb + L.lo_ln1_g), true));
    SS_TRY(upload_vec(st, W.ln1_b, 0, d, (float *)(lb + L.lo_ln1_b), ln));
    SS_TRY(upload_vec(st, W.ln2_g, 0, d, (float *)(lb + L.lo_ln2_g), true));
    SS_TRY(upload_vec(st, W.ln2_b, 0, d, (float *)(lb + L.lo_ln2_b), ln));
    const void *qkvw[3] = {W.wq, W.wk, W.wv};
    const void *qkvb[3] = {W.bq, W.bk, W.bv};
    for (int p = 0; p < 3; ++p) {
      SS_TRY(upload_matrix<T>(sh, st, qkvw[p], (size_t)Hp * Dh, 0, c0, d, HD, false, sh->wqkv[l].ptr, d / FK,
                              HD / 16, 1, p * (HD / 16)));
      SS_TRY(upload_vec(st, qkvb[p], c0, HD, bqkv + p * HD, bias));
    }
    SS_TRY(upload_matrix<T>(sh, st, W.wo, d, c0, 0, HD, d, false, sh->wo[l].ptr, HD / FK, d / 16, 1, 0));
    SS_TRY(upload_vec(st, W.bo, 0, d, bo, bias));
    if (m.act == SS_ACT_SWIGLU) {
      SS_TRY(upload_matrix<T>(sh, st, W.wg, Fp, 0, f0, d, L.Fs, false, sh->w1[l].ptr, d / FK, L.Fs / 16, 2, 0));
      SS_TRY(upload_matrix<T>(sh, st, W.wu, Fp, 0, f0, d, L.Fs, false, sh->w1[l].ptr, d / FK, L.Fs / 16, 2, 1));
    } else {
      SS_TRY(upload_matrix<T>(sh, st, W.w1, Fp, 0, f0, d, L.Fs, false, sh->w1[l].ptr, d / FK, L.Fs / 16, 1, 0));
      SS_TRY(upload_vec(st, W.b1, f0, L.Fs, b1, bias));
    }
    SS_TRY(upload_matrix<T>(sh, st, W.w2, d, f0, 0, L.Fs, d, false, sh->w2[l].ptr, L.Fs / FK, d / 16, 1, 0));
    SS_TRY(upload_vec(st, W.b2, 0, d, b2, bias));
    if (ln) {
      SS_TRY(launch_fold_norm(m.dtype, sh->wqkv[l].ptr, sh->wqkv[l].row_tiles, sh->wqkv[l].k_blocks, D.ln1_g, D.ln1_b, D.bqkv,
                              sh->wg_qkv[l], sh->cb_qkv[l], st));
      SS_TRY(launch_fold_norm(m.dtype, sh->w1[l].ptr, sh->w1[l].row_tiles, sh->w1[l].k_blocks, D.ln2_g, D.ln2_b, D.b1,
                              sh->wg_1[l], sh->cb_1[l], st));
    }
  }
  return SS_OK;
}

// what creation does after the model context is in place: RoPE table, empty cache, counters
static ss_status finish_create(Shard *sh, hipStream_t st, bool rope_in_place = false) {
  const Layout &L = sh->L;
  if (sh->m.pos == SS_POS_ROPE && !rope_in_place) {
    // angles in double on the host, table in float32
    std::vector<float2> tab((size_t)L.Smax * (L.Dh / 2));
    for (int p = 0; p < L.Smax; ++p)
      for (int i = 0; i < L.Dh / 2; ++i) {
        double ang = (double)p * pow((double)sh->m.rope_theta, -2.0 * i / L.Dh);
        tab[(size_t)p * (L.Dh / 2) + i] = make_float2((float)cos(ang), (float)sin(ang));
      }
    SS_HIP(hipMemcpyAsync(sh->rope, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice, st));
    SS_HIP(hipStreamSynchronize(st));
  }
  hipLaunchKernelGGL(fill_i32, dim3(1), dim3(32), 0, st, sh->d_len, 32, 0);
  hipLaunchKernelGGL(fill_i32, dim3(1), dim3(256), 0, st, (int32_t *)sh->zero_frag, 256, 0);
  const int nc = L.n_counters;
  hipLaunchKernelGGL(fill_i32, dim3(ceil_div(nc, 256)), dim3(256), 0, st, (int32_t *)(sh->ws + L.ws_counters), nc, 0);
  SS_HIP(hipGetLastError());
  SS_HIP(hipStreamSynchronize(st));
  return SS_OK;
}

}  // namespace ss

extern "C" {

ss_status ss_shard_create(const ss_model_desc *desc, const ss_slice *slice, const ss_weights *parent,
                          int32_t max_batch, int32_t max_seq, void *device_mem, size_t device_bytes,
                          void *hip_stream, ss_shard **out) {
  if (!desc || !slice || !parent || !device_mem || !out) SS_FAIL(SS_EINVAL, "NULL argument");
  *out = nullptr;
  SS_TRY(validate_desc(*desc, *slice, max_batch, max_seq));
  const ss_slice &ps = parent->slice;
  if (!(ps.layer_lo <= slice->layer_lo && slice->layer_hi <= ps.layer_hi && ps.head_lo <= slice->head_lo &&
        slice->head_hi <= ps.head_hi && ps.ffn_lo <= slice->ffn_lo && slice->ffn_hi <= ps.ffn_hi))
    SS_FAIL(SS_EINVAL, "slice is not inside the parent's slice");
  if (!parent->layers) SS_FAIL(SS_EINVAL, "parent->layers is NULL");
  if (((uintptr_t)device_mem) & 255) SS_FAIL(SS_EINVAL, "device_mem must be 256-byte aligned");
  Shard *sh = new (std::nothrow) Shard();
  if (!sh) SS_FAIL(SS_ENOMEM, "host allocation failed");
  sh->id = next_shard_id();
  sh->m = *desc;
  sh->s = *slice;
  compute_layout(*desc, *slice, max_batch, max_seq, &sh->L);
  const Layout &L = sh->L;
  if (device_bytes < L.total) {
    delete sh;
    SS_FAIL(SS_ENOMEM, "device_mem holds %zu bytes, the shard needs %zu", device_bytes, L.total);
  }
  hipStream_t st = (hipStream_t)hip_stream;
  sh->base = (char *)device_mem;
  bind_pointers(sh);
  sh->h_len.assign(max_batch, 0);
  ss_status rc = desc->dtype == SS_DTYPE_BF16 ? upload_all<bf16_t>(sh, parent, st) : upload_all<float>(sh, parent, st);
  if (rc == SS_OK) rc = finish_create(sh, st);
  if (rc != SS_OK) {
    delete sh;
    return rc;
  }
  *out = (ss_shard *)sh;
  return SS_OK;
}

size_t ss_shard_model_context_bytes(const ss_shard *shard) {
  return shard ? ((const Shard *)shard)->L.off_kv : 0;
}

ss_status ss_shard_destroy(ss_shard *shard) {
  if (!shard) return SS_OK;
  Shard *sh = (Shard *)shard;
  destroy_graphs(sh);
  delete sh;
  return SS_OK;
}

ss_status ss_shard_reset(ss_shard *shard, void *hip_stream) {
  if (!shard) SS_FAIL(SS_EINVAL, "NULL shard");
  Shard *sh = (Shard *)shard;
  hipLaunchKernelGGL(fill_i32, dim3(1), dim3(32), 0, (hipStream_t)hip_stream, sh->d_len, 32, 0);
  SS_HIP(hipGetLastError());
  std::fill(sh->h_len.begin(), sh->h_len.end(), 0);
  return SS_OK;
}

ss_status ss_committed_len(const ss_shard *shard, int32_t *out_host, void *hip_stream) {
  if (!shard || !out_host) SS_FAIL(SS_EINVAL, "NULL argument");
  const Shard *sh = (const Shard *)shard;
  SS_HIP(hipMemcpyAsync(out_host, sh->d_len, sh->L.Bmax * 4, hipMemcpyDeviceToHost, (hipStream_t)hip_stream));
  SS_HIP(hipStreamSynchronize((hipStream_t)hip_stream));
  return SS_OK;
}

ss_status ss_shard_geometry(const ss_shard *shard, int32_t out[6]) {
  if (!shard || !out) SS_FAIL(SS_EINVAL, "NULL argument");
  const Shard *sh = (const Shard *)shard;
  out[0] = sh->L.Ls, out[1] = sh->L.Hs, out[2] = sh->L.Fs, out[3] = sh->L.Bmax, out[4] = sh->L.Smax, out[5] = sh->L.esz;
  return SS_OK;
}

ss_status ss_debug_interrupt_after_layer(ss_shard *shard, int32_t layer) {
  if (!shard) SS_FAIL(SS_EINVAL, "NULL shard");
  Shard *sh = (Shard *)shard;
  if (layer < -1 || layer >= sh->L.Ls) SS_FAIL(SS_EINVAL, "layer %d outside the shard's %d layers", layer, sh->L.Ls);
  sh->interrupt_after = layer;
  return SS_OK;
}

ss_status ss_set_graph_launch(ss_shard *shard, int32_t enabled) {
  if (!shard) SS_FAIL(SS_EINVAL, "NULL shard");
  ((Shard *)shard)->use_graph = enabled != 0;
  return SS_OK;
}

// ---------------------------------------------------------------------------
// a shard whose model context comes from resident shards
// ---------------------------------------------------------------------------
ss_status ss_shard_create_from_resident(const ss_model_desc *desc, const ss_slice *slice, ss_shard *const *sources,
                                        int32_t n_sources, int32_t max_batch, int32_t max_seq, void *device_mem,
                                        size_t device_bytes, void *hip_stream, ss_shard **out, uint64_t *bytes_copied) {
  if (!desc || !slice || !sources || n_sources < 1 || !device_mem || !out) SS_FAIL(SS_EINVAL, "NULL argument");
  *out = nullptr;
  SS_TRY(validate_desc(*desc, *slice, max_batch, max_seq));
  if (((uintptr_t)device_mem) & 255) SS_FAIL(SS_EINVAL, "device_mem must be 256-byte aligned");
  std::vector<const Shard *> src(n_sources);
  for (int i = 0; i < n_sources; ++i) {
    src[i] = (const Shard *)sources[i];
    if (!src[i]) SS_FAIL(SS_EINVAL, "sources[%d] is NULL", i);
    const ss_model_desc &o = src[i]->m;
    if (o.n_layers != desc->n_layers || o.d_model != desc->d_model || o.n_heads != desc->n_heads ||
        o.head_dim != desc->head_dim || o.ffn != desc->ffn || o.vocab != desc->vocab || o.max_pos != desc->max_pos ||
        o.norm != desc->norm || o.act != desc->act || o.pos != desc->pos || o.has_bias != desc->has_bias ||
        o.dtype != desc->dtype)
      SS_FAIL(SS_EINVAL, "sources[%d] holds another model", i);
  }
  Shard *sh = new (std::nothrow) Shard();
  if (!sh) SS_FAIL(SS_ENOMEM, "host allocation failed");
  sh->id = next_shard_id();
  sh->m = *desc, sh->s = *slice;
  compute_layout(*desc, *slice, max_batch, max_seq, &sh->L);
  const Layout &L = sh->L;
  if (device_bytes < L.total) {
    delete sh;
    SS_FAIL(SS_ENOMEM, "device_mem holds %zu bytes, the shard needs %zu", device_bytes, L.total);
  }
  sh->base = (char *)device_mem;
  bind_pointers(sh);
  sh->h_len.assign(max_batch, 0);
  hipStream_t st = (hipStream_t)hip_stream;
  const int d = L.d, Dh = L.Dh, esz = L.esz, FK = esz == 2 ? 32 : 16;
  const bool ln = desc->norm == SS_NORM_LAYERNORM, glu = desc->act == SS_ACT_SWIGLU, bias = desc->has_bias != 0;

  std::vector<Copy2D> jobs;
  uint64_t total_bytes = 0;
  auto add = [&](const void *s_, void *d_, uint32_t rows, size_t row_bytes, size_t s_stride, size_t d_stride) {
    if (!rows || !row_bytes) return;
    // one run of many bytes is as good as rows of 64 KiB
    if (rows == 1 && row_bytes > 65536) {
      const uint32_t full = (uint32_t)(row_bytes / 65536);
      const size_t rest = row_bytes - (size_t)full * 65536;
      jobs.push_back(Copy2D{(const char *)s_, (char *)d_, 65536, 65536, full, 65536, 1, 1, 0, 0});
      if (rest) jobs.push_back(Copy2D{(const char *)s_ + (size_t)full * 65536, (char *)d_ + (size_t)full * 65536, 0, 0, 1, (uint32_t)rest, 1, 1, 0, 0});
    } else {
      jobs.push_back(Copy2D{(const char *)s_, (char *)d_, s_stride, d_stride, rows, (uint32_t)row_bytes, 1, 1, 0, 0});
    }
    total_bytes += (uint64_t)rows * row_bytes;
  };
  ss_status rc = SS_OK;
  auto fail = [&](const char *what, int l) {
    set_error("the sources do not hold %s of layer %d that the new slice needs", what, l);
    rc = SS_EINVAL;
  };

  // replicated context from the first source
  const Shard *s0 = src[0];
  add(s0->wte, sh->wte, 1, (size_t)L.V * d * esz, 0, 0);
  if (L.max_pos) add(s0->wpe, sh->wpe, 1, (size_t)L.max_pos * d * esz, 0, 0);
  add(s0->lm_head.ptr, sh->lm_head.ptr, 1, (size_t)sh->lm_head.row_tiles * sh->lm_head.k_blocks * 1024, 0, 0);
  add(s0->lnf_g, sh->lnf_g, 1, (size_t)d * 4, 0, 0);
  if (ln) {
    add(s0->lnf_b, sh->lnf_b, 1, (size_t)d * 4, 0, 0);
    add(s0->wg_lm, sh->wg_lm, 1, align_up((size_t)L.V, 16) * 4, 0, 0);
    add(s0->cb_lm, sh->cb_lm, 1, align_up((size_t)L.V, 16) * 4, 0, 0);
  }
  // the rotation table is indexed by position: a source's table covers ours if it is as long
  bool rope_copied = false;
  if (desc->pos == SS_POS_ROPE && s0->L.Smax >= L.Smax && s0->m.rope_theta == desc->rope_theta) {
    add(s0->rope, sh->rope, 1, (size_t)L.Smax * (Dh / 2) * sizeof(float2), 0, 0);
    rope_copied = true;
  }
  const int kbd = d / FK;  // k blocks of a d-long reduction
  for (int l = 0; l < L.Ls && rc == SS_OK; ++l) {
    const int gl = slice->layer_lo + l;  // layer of the model
    char *lb = sh->base + L.off_layer[l];
    bool vectors_done = false, progress = true;
    int heads_done = 0, cols_done = 0;
    // sources in any order: keep passing over them while one of them extends the covered prefix
    while (progress && rc == SS_OK && (heads_done < L.Hs || cols_done < L.Fs || !vectors_done)) {
    progress = false;
    for (const Shard *q : src) {
      if (gl < q->s.layer_lo || gl >= q->s.layer_hi) continue;
      const Layout &Q = q->L;
      const char *qb = q->base + Q.off_layer[gl - q->s.layer_lo];
      if (!vectors_done) {  // replicated vectors of the layer
        add(qb + Q.lo_ln1_g, lb + L.lo_ln1_g, 1, (size_t)d * 4, 0, 0);
        add(qb + Q.lo_ln2_g, lb + L.lo_ln2_g, 1, (size_t)d * 4, 0, 0);
        if (ln) add(qb + Q.lo_ln1_b, lb + L.lo_ln1_b, 1, (size_t)d * 4, 0, 0), add(qb + Q.lo_ln2_b, lb + L.lo_ln2_b, 1, (size_t)d * 4, 0, 0);
        if (bias) add(qb + Q.lo_bo, lb + L.lo_bo, 1, (size_t)d * 4, 0, 0), add(qb + Q.lo_b2, lb + L.lo_b2, 1, (size_t)d * 4, 0, 0);
        vectors_done = progress = true;
      }
      // heads the source adds to what is already covered (sources are taken in order; heads
      // must come as a contiguous run continuing the covered prefix)
      const int h0 = std::max(slice->head_lo + heads_done, q->s.head_lo), h1 = std::min(slice->head_hi, q->s.head_hi);
      if (h0 == slice->head_lo + heads_done && h1 > h0) {
        const int nh = h1 - h0, hs = h0 - q->s.head_lo, hd = h0 - slice->head_lo;
        const size_t head_frag_bytes = (size_t)(Dh / 16) * kbd * 1024;  // one head's tiles of one of q, k, v
        for (int p = 0; p < 3; ++p) {
          add(qb + Q.lo_wqkv + ((size_t)p * Q.Hs + hs) * head_frag_bytes, lb + L.lo_wqkv + ((size_t)p * L.Hs + hd) * head_frag_bytes,
              1, (size_t)nh * head_frag_bytes, 0, 0);
          if (bias) add(qb + Q.lo_bqkv + ((size_t)p * Q.Hs + hs) * Dh * 4, lb + L.lo_bqkv + ((size_t)p * L.Hs + hd) * Dh * 4, 1, (size_t)nh * Dh * 4, 0, 0);
          if (ln) {
            add(qb + Q.lo_wg_qkv + ((size_t)p * Q.Hs + hs) * Dh * 4, lb + L.lo_wg_qkv + ((size_t)p * L.Hs + hd) * Dh * 4, 1, (size_t)nh * Dh * 4, 0, 0);
            add(qb + Q.lo_cb_qkv + ((size_t)p * Q.Hs + hs) * Dh * 4, lb + L.lo_cb_qkv + ((size_t)p * L.Hs + hd) * Dh * 4, 1, (size_t)nh * Dh * 4, 0, 0);
          }
        }
        // output projection: every row tile, the k blocks of these heads
        const size_t hk = (size_t)(Dh / FK) * 1024;  // one head's k blocks of one row tile
        add(qb + Q.lo_wo + hs * hk, lb + L.lo_wo + hd * hk, d / 16, nh * hk, (size_t)Q.Hs * hk, (size_t)L.Hs * hk);
        heads_done += nh;
        progress = true;
      }
      const int f0 = std::max(slice->ffn_lo + cols_done, q->s.ffn_lo), f1 = std::min(slice->ffn_hi, q->s.ffn_hi);
      if (f0 == slice->ffn_lo + cols_done && f1 > f0) {
        const int nf = f1 - f0, fs = f0 - q->s.ffn_lo, fd = f0 - slice->ffn_lo;
        if (nf % 64 || fs % 64 || fd % 64) {
          set_error("FFN columns shared with a source must come in multiples of 64");
          rc = SS_EINVAL;
          break;
        }
        const int c1 = glu ? 2 : 1;  // gate/up tiles are interleaved: two tiles per 16 columns
        add(qb + Q.lo_w1 + (size_t)(fs / 16) * c1 * kbd * 1024, lb + L.lo_w1 + (size_t)(fd / 16) * c1 * kbd * 1024, 1,
            (size_t)(nf / 16) * c1 * kbd * 1024, 0, 0);
        if (bias && !glu) add(qb + Q.lo_b1 + (size_t)fs * 4, lb + L.lo_b1 + (size_t)fd * 4, 1, (size_t)nf * 4, 0, 0);
        if (ln) {
          add(qb + Q.lo_wg_1 + (size_t)fs * c1 * 4, lb + L.lo_wg_1 + (size_t)fd * c1 * 4, 1, (size_t)nf * c1 * 4, 0, 0);
          add(qb + Q.lo_cb_1 + (size_t)fs * c1 * 4, lb + L.lo_cb_1 + (size_t)fd * c1 * 4, 1, (size_t)nf * c1 * 4, 0, 0);
        }
        const size_t fk = 1024;  // one k block of one row tile
        add(qb + Q.lo_w2 + (size_t)(fs / FK) * fk, lb + L.lo_w2 + (size_t)(fd / FK) * fk, d / 16, (size_t)(nf / FK) * fk,
            (size_t)(Q.Fs / FK) * fk, (size_t)(L.Fs / FK) * fk);
        cols_done += nf;
        progress = true;
      }
    }
    }
    if (rc != SS_OK) break;
    if (!vectors_done) fail("the norm vectors", gl);
    else if (heads_done != L.Hs) fail("all the heads", gl);
    else if (cols_done != L.Fs) fail("all the FFN columns", gl);
  }
  // the descriptors go through the new shard's own workspace
  if (rc == SS_OK) {
    uint32_t blocks = 0;
    for (Copy2D &c : jobs) {
      if (c.row_bytes % 16 || ((uintptr_t)c.src & 15) || ((uintptr_t)c.dst & 15) || c.src_stride % 16 || c.dst_stride % 16) {
        set_error("internal: a re-slice copy is not 16-byte aligned");
        rc = SS_EINVAL;
        break;
      }
      c.first_block = blocks;
      if (c.row_bytes >= 16384) {  // pieces of 16 KiB: four vectors a thread, requested together (smaller pieces copy faster, but every block finds its descriptor by bisection)
        c.rows_per_block = 1, c.blocks_per_row = (uint32_t)ceil_div((int)(c.row_bytes >> 4), 1024);
        blocks += c.rows * c.blocks_per_row;
      } else {
        c.rows_per_block = std::max<uint32_t>(2, 16384 / c.row_bytes), c.blocks_per_row = 1;
        blocks += (c.rows + c.rows_per_block - 1) / c.rows_per_block;
      }
    }
    if (rc == SS_OK && jobs.size() * sizeof(Copy2D) > L.ws_bytes) {
      set_error("re-slice: %zu copy descriptors do not fit the workspace", jobs.size());
      rc = SS_EINVAL;
    }
    if (rc == SS_OK) {
      hipError_t e = hipMemcpyAsync(sh->ws, jobs.data(), jobs.size() * sizeof(Copy2D), hipMemcpyHostToDevice, st);
      if (e == hipSuccess) {
        hipLaunchKernelGGL(copy2d_kernel, dim3(blocks), dim3(256), 0, st, (const Copy2D *)sh->ws, (int)jobs.size());
        e = hipGetLastError();
      }
      if (e == hipSuccess) e = hipStreamSynchronize(st);  // the host descriptor array dies with this call
      if (e != hipSuccess) {
        set_error("re-slice: %s", hipGetErrorString(e));
        rc = SS_EHIP;
      }
    }
  }
  if (rc == SS_OK) rc = finish_create(sh, st, rope_copied);
  if (rc != SS_OK) {
    delete sh;
    return rc;
  }
  if (bytes_copied) *bytes_copied = total_bytes;
  *out = (ss_shard *)sh;
  return SS_OK;
}

// ---------------------------------------------------------------------------
// re-partition
// ---------------------------------------------------------------------------
ss_status ss_kv_repack(ss_shard *dst_, const ss_shard *src_, const int32_t *batch_map, int32_t first_source,
                       uint64_t *bytes_moved, void *hip_stream) {
  if (!dst_ || !src_ || !batch_map) SS_FAIL(SS_EINVAL, "NULL argument");
  Shard *dst = (Shard *)dst_;
  const Shard *src = (const Shard *)src_;
  if (dst == src) SS_FAIL(SS_EINVAL, "source and destination are the same shard");
  if (dst->L.esz != src->L.esz || dst->L.Dh != src->L.Dh || dst->m.kv_dtype != src->m.kv_dtype)
    SS_FAIL(SS_EINVAL, "source and destination differ in cache dtype or head_dim");
  RepackArgs a;
  memset(&a, 0, sizeof(a));
  bool used[32] = {false};
  int max_len = 0;
  uint64_t rows_total = 0;
  for (int bd = 0; bd < dst->L.Bmax; ++bd) {
    int bs = batch_map[bd];
    if (bs < 0) continue;
    if (bs >= src->L.Bmax) SS_FAIL(SS_EINVAL, "batch_map[%d] = %d outside the source's %d rows", bd, bs, src->L.Bmax);
    if (used[bs]) SS_FAIL(SS_EINVAL, "source row %d mapped twice", bs);
    used[bs] = true;
    int n = src->h_len[bs];
    if (n > dst->L.Smax) SS_FAIL(SS_ESTATE, "source row %d holds %d rows, destination capacity is %d", bs, n, dst->L.Smax);
    if (!first_source && dst->h_len[bd] != n)
      SS_FAIL(SS_ESTATE, "destination row %d already holds %d rows, this source has %d", bd, dst->h_len[bd], n);
    a.map_dst[a.n_map] = bd, a.map_src[a.n_map] = bs, a.map_len[a.n_map] = n;
    a.n_map++;
    max_len = std::max(max_len, n);
    rows_total += (uint64_t)n;
  }
  const int l_lo = std::max(dst->s.layer_lo, src->s.layer_lo), l_hi = std::min(dst->s.layer_hi, src->s.layer_hi);
  const int h_lo = std::max(dst->s.head_lo, src->s.head_lo), h_hi = std::min(dst->s.head_hi, src->s.head_hi);
  a.n_layers = std::max(0, l_hi - l_lo);
  a.n_heads = std::max(0, h_hi - h_lo);
  a.row_bytes = dst->L.Dh * dst->L.esz;
  if (bytes_moved) *bytes_moved = (uint64_t)a.n_layers * 2 * a.n_heads * rows_total * a.row_bytes;
  for (int i = 0; i < a.n_map; ++i) dst->h_len[a.map_dst[i]] = a.map_len[i];
  if (a.n_map == 0) return SS_OK;
  a.dst_len = dst->d_len;
  hipStream_t st = (hipStream_t)hip_stream;
  if (a.n_layers == 0 || a.n_heads == 0 || max_len == 0) {  // nothing to move: only the lengths change
    hipLaunchKernelGGL(kv_repack_commit, dim3(1), dim3(32), 0, st, a);
    SS_HIP(hipGetLastError());
    return SS_OK;
  }
  a.src = src->kv_ptr(l_lo - src->s.layer_lo, 0) + (size_t)(h_lo - src->s.head_lo) * src->kv_head_stride();
  a.dst = dst->kv_ptr(l_lo - dst->s.layer_lo, 0) + (size_t)(h_lo - dst->s.head_lo) * dst->kv_head_stride();
  a.s_layer = src->kv_layer_stride(), a.s_plane = src->kv_plane_stride(), a.s_row = src->kv_row_stride(),
  a.s_head = src->kv_head_stride();
  a.d_layer = dst->kv_layer_stride(), a.d_plane = dst->kv_plane_stride(), a.d_row = dst->kv_row_stride(),
  a.d_head = dst->kv_head_stride();
  const size_t seg_vec = ((size_t)max_len * a.row_bytes) >> 4;
  a.chunk_vec = 256;  // 4 KiB per block, one vector per thread
  a.chunks_per_seg = (int)((seg_vec + a.chunk_vec - 1) / a.chunk_vec);
  const size_t gy = (size_t)a.n_map * a.n_heads, gz = (size_t)a.n_layers * 2;
  if (gy > 65535 || gz > 65535 || (size_t)a.chunks_per_seg > 0x7fffffffULL) SS_FAIL(SS_EINVAL, "re-partition too large for one launch");
  hipLaunchKernelGGL(kv_repack_kernel, dim3((unsigned)a.chunks_per_seg, (unsigned)gy, (unsigned)gz), dim3(256), 0, st, a);
  hipLaunchKernelGGL(kv_repack_commit, dim3(1), dim3(32), 0, st, a);
  SS_HIP(hipGetLastError());
  return SS_OK;
}

// ---------------------------------------------------------------------------
// export / import in the exchange order [layer][K|V][b][head][j < n[b]][Dh]
// ---------------------------------------------------------------------------
size_t ss_kv_export_bytes(const ss_shard *shard) {
  if (!shard) return 0;
  const Shard *sh = (const Shard *)shard;
  size_t rows = 0;
  for (int b = 0; b < sh->L.Bmax; ++b) rows += sh->h_len[b];
  return (size_t)sh->L.Ls * 2 * sh->L.Hs * rows * sh->L.Dh * sh->L.esz;
}

static ss_status kv_transfer(const Shard *sh, char *host, size_t bytes, const int32_t *lens, bool to_host,
                             hipStream_t st) {
  size_t rows = 0;
  for (int b = 0; b < sh->L.Bmax; ++b) rows += lens[b];
  size_t need = (size_t)sh->L.Ls * 2 * sh->L.Hs * rows * sh->L.Dh * sh->L.esz;
  if (bytes != need) SS_FAIL(SS_EINVAL, "buffer holds %zu bytes, the committed rows take %zu", bytes, need);
  const size_t rb = (size_t)sh->L.Dh * sh->L.esz;
  size_t off = 0;
  for (int l = 0; l < sh->L.Ls; ++l)
    for (int c = 0; c < 2; ++c)
      for (int b = 0; b < sh->L.Bmax; ++b) {
        size_t w = (size_t)lens[b] * rb;  // bytes per head for this row
        if (!w) continue;
        char *dev = sh->kv_ptr(l, c) + b * sh->kv_row_stride();
        if (to_host)
          SS_HIP(hipMemcpy2DAsync(host + off, w, dev, sh->kv_head_stride(), w, sh->L.Hs, hipMemcpyDeviceToHost, st));
        else
          SS_HIP(hipMemcpy2DAsync(dev, sh->kv_head_stride(), host + off, w, w, sh->L.Hs, hipMemcpyHostToDevice, st));
        off += w * sh->L.Hs;
      }
  SS_HIP(hipStreamSynchronize(st));
  return SS_OK;
}

ss_status ss_kv_export(const ss_shard *shard, void *host_dst, size_t bytes, void *hip_stream) {
  if (!shard || (!host_dst && bytes)) SS_FAIL(SS_EINVAL, "NULL argument");
  const Shard *sh = (const Shard *)shard;
  return kv_transfer(sh, (char *)host_dst, bytes, sh->h_len.data(), true, (hipStream_t)hip_stream);
}

ss_status ss_kv_import(ss_shard *shard, const void *host_src, const int32_t *lens, size_t bytes, void *hip_stream) {
  if (!shard || !lens || (!host_src && bytes)) SS_FAIL(SS_EINVAL, "NULL argument");
  Shard *sh = (Shard *)shard;
  for (int b = 0; b < sh->L.Bmax; ++b)
    if (lens[b] < 0 || lens[b] > sh->L.Smax) SS_FAIL(SS_EINVAL, "lens[%d] = %d outside [0,%d]", b, lens[b], sh->L.Smax);
  SS_TRY(kv_transfer(sh, (char *)host_src, bytes, lens, false, (hipStream_t)hip_stream));
  SS_HIP(hipMemcpyAsync(sh->d_len, lens, sh->L.Bmax * 4, hipMemcpyHostToDevice, (hipStream_t)hip_stream));
  SS_HIP(hipStreamSynchronize((hipStream_t)hip_stream));
  for (int b = 0; b < sh->L.Bmax; ++b) sh->h_len[b] = lens[b];
  return SS_OK;
}

}  // extern "C"
