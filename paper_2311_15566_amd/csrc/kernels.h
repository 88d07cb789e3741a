// Launchers of the hot-path kernels.  Every launcher checks on the host that the operand
// shapes fit what its kernel assumes before it launches.
#pragma once
#include "common.h"

namespace ss {

enum Prologue { PRO_ACT = 0, PRO_NORM = 1 };
enum Epilogue { EPI_F32 = 0, EPI_RESID = 1, EPI_ACT = 2, EPI_SWIGLU = 3, EPI_LOGITS = 4 };

// Skinny GEMM of the decode step: out[b, n] = sum_k act[b, k] * W[n, k], b < B <= 32.
// HBM-bound weight streaming: each wave streams whole 1 KiB weight fragments, activations are
// staged once per block in LDS, split-K partials are reduced by the last block to arrive
// (fixed order, so results do not depend on scheduling).
struct SkinnyArgs {
  // weights
  const void *w;
  int tasks;      // wave tasks: 16-row tiles (SwiGLU: gate/up tile pairs)
  int k_blocks;   // fragments along K
  int split;      // blocks along K
  int kb_per_split;
  int lds_chunk;  // fragments staged in LDS at a time
  int B;          // live batch rows
  int nb;         // 16-row batch tiles (1 or 2)
  int N;          // logical output features (for masking)
  // prologue
  const void *act;      // PRO_ACT: fragments [nb][k_blocks]
  const float *x;       // PRO_NORM: [B][K] float32, row-major
  const float *stats;   // PRO_NORM: [32][2] = (mean, 1/std)
  const float *gamma, *beta;
  // split-K scratch
  float *splitk;
  int *counters;        // [groups] + 1
  // epilogues
  const float *bias;
  float *out_f32;       // EPI_F32 / EPI_LOGITS: [B][ld_out]
  int ld_out;
  const float *x_in;    // EPI_RESID: residual stream before this GEMM, [B][N]
  float *x_resid;       // EPI_RESID: residual stream after it (may equal x_in only when no other block of the
                        // same launch reads it)
  float *stat_part;     // EPI_RESID: [groups][32][2]
  float *stats_out;     // EPI_RESID: [32][2]
  int rms;              // EPI_RESID: statistics for RMSNorm (no mean)
  float eps;
  void *act_out;        // EPI_ACT / EPI_SWIGLU: fragments [nb][out_k_blocks]
  int out_k_blocks;
  int act_kind;
  float *am_val;        // EPI_LOGITS: [groups][32]
  int *am_idx;
  int32_t *next_tokens;
  int32_t *lens[8];     // EPI_LOGITS: committed lengths to advance (all shards of the group)
  int n_lens;
  int commit_inc;
};
ss_status launch_skinny(int dtype, int pro, int epi, const SkinnyArgs &a, hipStream_t st);
ss_status check_skinny(int dtype, const SkinnyArgs &a);  // the shape checks launch_skinny makes
// fills split / kb_per_split / lds_chunk / nb from the shape
// (target_blocks = 0: the default of the kernel-by-kernel path; < 0: plan for the persistent kernel
// with -target_blocks resident blocks)
void plan_skinny(SkinnyArgs *a, int esz, size_t splitk_bytes, int weight_tiles_per_wave, int target_blocks);

// Prefill GEMM: out[t, n] = sum_k act[t, k] * W[n, k] over T tokens (multiple of 128), MFMA-bound.
struct TileGemmArgs {
  const void *w;      // weight fragments
  int row_tiles;      // 16-row weight tiles (SwiGLU: 2 per 16 outputs, interleaved)
  int k_blocks;
  const void *act;    // activation fragments [T/16][k_blocks][act_parts]
  int act_parts;      // 1, or 2 for bf16 hi/lo pairs
  int T;              // tokens (padded to 128)
  int T_live;         // tokens that exist
  int N;
  const float *bias;
  float *out_f32;     // EPI_F32: [T][ld_out]
  int ld_out;
  float *x_resid;     // EPI_RESID: [T][N]
  void *act_out;      // EPI_ACT / EPI_SWIGLU: fragments [T/16][out_k_blocks][out_parts]
  int out_k_blocks;
  int out_parts;
  int act_kind;
};
ss_status launch_tile_gemm(int dtype, int epi, const TileGemmArgs &a, hipStream_t st);

// Decode attention over the committed cache (plus the new token), sequence-split.
struct DecodeAttnArgs {
  const float *qkv;     // [B][3*Hs*Dh] float32: q | k | v of the new token, biases applied
  char *k_cache, *v_cache;   // this layer's planes: [Bmax][Hs][Smax][Dh]
  size_t row_stride, head_stride;  // bytes
  const int32_t *lens;  // committed lengths (device)
  const float2 *rope;   // [Smax][Dh/2] or NULL
  float *part;          // [B*Hs][splits][Dh+4]
  int *counters;        // [B*Hs]
  void *o_out;          // fragments [nb][Hs*Dh / FragK]
  int B, Hs, Dh, Smax;
  int kv_dtype;         // cache element type (SS_DTYPE_*)
  int rows_per_block, splits;
};
ss_status launch_decode_attn(int dtype, const DecodeAttnArgs &a, hipStream_t st);
ss_status check_decode_attn(const DecodeAttnArgs &a);

// One phase of the decode step: a kernel of the kernel-by-kernel path, or one stretch between
// two device-wide barriers of the persistent kernel.
enum PhaseKind { PH_EMBED = 0, PH_QKV = 1, PH_ATTN = 2, PH_RESID = 3, PH_FFN_UP = 4, PH_LM_HEAD = 5 };
struct EmbedArgs {
  const int32_t *tokens;  // [rows]
  const void *wte, *wpe;  // [V][d], [max_pos][d] or NULL
  const int32_t *lens;    // decode: position = committed length; NULL: position = row % S
  int S;
  float *x;               // [rows][d]
  float *stats;           // [rows][2] (mean, 1/std) of the first norm, or NULL
  int d, V, rms;
  float eps;
};

struct Phase {
  int kind;      // PhaseKind; also the timing class
  int gx, gy;    // blocks: (rows, 1), (groups, splits) or (batch*heads, splits)
  int shard;     // index of the shard in the group that owns the phase's scratch
  EmbedArgs e;
  SkinnyArgs g;
  DecodeAttnArgs at;
};

// Prefill: rotate q, k; write K/V rows [0, S) of every sequence; then causal attention.
struct PrefillAttnArgs {
  float *qkv;           // [T][3*Hs*Dh] float32 (q rotated in place)
  char *k_cache, *v_cache;
  size_t row_stride, head_stride;
  const float2 *rope;
  void *o_out;          // fragments [T/16][Hs*Dh / FragK][parts of the operand type]
  int B, S, Hs, Dh, Smax;
  int kv_dtype;
};
ss_status launch_prefill_kv_write(int dtype, const PrefillAttnArgs &a, hipStream_t st);
ss_status launch_prefill_attn(int dtype, const PrefillAttnArgs &a, hipStream_t st);

}  // namespace ss
