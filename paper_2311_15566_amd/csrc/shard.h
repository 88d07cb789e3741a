// Host object of one shard and the carve-up of its device memory.
#pragma once
#include <tuple>

#include "kernels.h"

namespace ss {

// One weight matrix in matrix-core operand order (see frag_offset).
struct FragMat {
  void *ptr = nullptr;
  int rows = 0;        // logical output features (SwiGLU w1: 2*Fs, gate/up tiles interleaved)
  int K = 0;           // logical reduction length
  int row_tiles = 0;   // ceil(rows/16)
  int k_blocks = 0;    // ceil(K/FragK)
};

struct Layout {
  // sizes
  int Ls, Hs, Fs, d, Dh, V, max_pos, Bmax, Smax;
  int esz;             // bytes per element of the model dtype
  int Bpad;            // max_batch rounded up to 16
  int Tmax;            // prefill tokens the workspace holds (Bmax*Smax rounded up to 256, the prefill GEMM's token block)
  int qkv_n;           // 3*Hs*Dh
  int w1_rows;         // Fs or 2*Fs
  int attn_splits;     // sequence splits of decode attention at Smax
  bool two_part_qk;    // initial phase: the q and k columns of the q|k|v GEMM take a two-part (high + low halves) operand
  // offsets into device_mem
  size_t off_wte, off_wpe, off_lm, off_lnf_g, off_lnf_b, off_rope;
  std::vector<size_t> off_layer;       // start of each layer's block
  size_t layer_bytes;
  size_t lo_ln1_g, lo_ln1_b, lo_ln2_g, lo_ln2_b, lo_wqkv, lo_bqkv, lo_wo, lo_bo, lo_w1, lo_b1, lo_w2, lo_b2;
  size_t lo_wg_qkv, lo_cb_qkv, lo_wg_1, lo_cb_1;  // gamma / beta+bias folded into the QKV and first FFN matrices
  size_t off_wg_lm, off_cb_lm;
  size_t off_kv, kv_bytes, off_len, off_zero;  // off_zero: 1 KiB of zeros (an operand fragment of nothing)
  size_t off_ws, ws_bytes;             // workspace, doubles as upload staging
  // workspace sub-offsets (relative to off_ws)
  size_t ws_x, ws_a, ws_a_lo, ws_qkv, ws_o, ws_u, ws_counters, ws_attn_part, ws_argmax;  // ws_a_lo: low parts of the q|k|v operand of the initial phase (two_part_qk), else unused
  size_t ws_vt;        // initial phase: one layer's values transposed, [Bmax*Hs][Dh][Smax rounded up to 64] halves
  size_t ws_pstat;     // initial phase: partial row sums [2 * ceil(d / 128)][Tmax] float2, then (mean, rstd, mean - centre, -) [Tmax] float4
  int n_counters;
  // decode step (rows = batch): residual stream [32][d] f32, operand of the next normalised GEMM
  // ((x - c) * gamma), partial row sums [d/16][32][2], the rows' centres [32], q|k|v [32][qkv_n] f32,
  // attention output and FFN activation operands
  size_t ws_xd, ws_ad, ws_statd, ws_cen, ws_qkvd, ws_od, ws_ud;
  size_t ws_ffnpart, ffnpart_bytes;  // partial outputs of a first FFN matrix whose K is cut into slices (more than 16 batch rows, no gate): [kQkvParts][32][Fs] float32, else 0 bytes
  size_t ws_dec_end;   // the decode step's scratch is workspace bytes [ws_xd, ws_dec_end): the buffers above, then
                       // the attention counters and partials and the LM head's candidates
  size_t total;
};

bool compute_layout(const ss_model_desc &m, const ss_slice &s, int max_batch, int max_seq, Layout *L);

// What a captured decode step depends on: the caller's buffers and stream, the batch size, the
// identity of every shard of the group (a process-unique id, not the host address, which the
// allocator hands out again after a destroy) and the launch-shape epoch (bumped whenever the shapes
// the plan builder would choose may have changed).
struct GraphKey {
  std::vector<const void *> ptrs;
  std::vector<uint64_t> ids;
  uint64_t epoch;
  int B;
  bool operator<(const GraphKey &o) const {
    return std::tie(B, epoch, ids, ptrs) < std::tie(o.B, o.epoch, o.ids, o.ptrs);
  }
};

struct Shard {
  uint64_t id = 0;       // process-unique, never reused
  ss_model_desc m;
  ss_slice s;
  Layout L;
  char *base = nullptr;  // device_mem
  // model context
  void *wte = nullptr, *wpe = nullptr;
  FragMat lm_head;
  float *lnf_g = nullptr, *lnf_b = nullptr;
  float2 *rope = nullptr;  // [Smax][Dh/2] (cos, sin)
  std::vector<LayerDev> layers;
  std::vector<FragMat> wqkv, wo, w1, w2;
  // folded norm vectors of the decode GEMMs (NULL where the model has none)
  std::vector<float *> wg_qkv, cb_qkv, wg_1, cb_1;
  float *wg_lm = nullptr, *cb_lm = nullptr;
  // cache context
  char *kv = nullptr;      // [Ls][2][Bmax][Hs][Smax][Dh]
  int32_t *d_len = nullptr;
  void *zero_frag = nullptr;
  std::vector<int32_t> h_len;  // host mirror of the committed lengths
  // workspace
  char *ws = nullptr;
  char *dec = nullptr;   // where the decode step's scratch starts: ws + L.ws_xd, unless a call puts it elsewhere
  char *dec_at(size_t ws_off) const { return dec + (ws_off - L.ws_xd); }  // a decode-scratch buffer by its workspace offset
  int interrupt_after = -1;
  bool use_graph = true;
  std::map<GraphKey, hipGraphExec_t> graphs;
  // per-kernel-class event timing (measurement aid)
  bool timing = false;
  struct TimedLaunch { int cls; hipEvent_t e0, e1; };
  std::vector<TimedLaunch> timed;
  std::vector<hipEvent_t> free_events;

  size_t kv_head_stride() const { return (size_t)L.Smax * L.Dh * L.esz; }  // bytes between heads
  size_t kv_row_stride() const { return kv_head_stride() * L.Hs; }          // between batch rows
  size_t kv_plane_stride() const { return kv_row_stride() * L.Bmax; }       // between K and V
  size_t kv_layer_stride() const { return kv_plane_stride() * 2; }
  char *kv_ptr(int layer, int c) const { return kv + layer * kv_layer_stride() + c * kv_plane_stride(); }
};

// shard.hip
ss_status validate_desc(const ss_model_desc &m, const ss_slice &s, int max_batch, int max_seq);
void bind_pointers(Shard *sh);  // every device pointer of the shard from base + layout

// decode.hip
ss_status run_decode_step(Shard *const *group, int n_group, const int32_t *tokens_in, const float *hidden_in, int B,
                          float *hidden_out, float *logits, int32_t *next_tokens, hipStream_t st,
                          int stop_after_layer);
ss_status run_prefill(Shard *const *group, int n_group, const int32_t *tokens, const float *hidden_in, int B, int S_in,
                      float *hidden_out, float *logits, int32_t *next_tokens, hipStream_t st);
void destroy_graphs(Shard *sh);
uint64_t next_shard_id();

}  // namespace ss
