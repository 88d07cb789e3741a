// Launchers of the hot-path kernels.  Every launcher checks on the host that the operand
// shapes fit what its kernel assumes before it launches.
#pragma once
#include "common.h"

namespace ss {

enum Epilogue { EPI_F32 = 0, EPI_RESID = 1, EPI_ACT = 2, EPI_SWIGLU = 3, EPI_LOGITS = 4 };
constexpr int kQkvParts = 8;  // partial q|k|v sums a decode step's workspace holds (slices the q|k|v GEMM may cut K into)

// Element type of both operands of the GEMMs for a model of element type T.  bf16 models: halves.
// Activations need more than bf16's 8 significant bits to stay under the logits bar, a half has 11;
// the matrix cores take both operands in one type, so the weight fragments are stored as halves too
// (converted at upload: exact for magnitudes from 2^-17 up, an 8-bit significand fits into 11 bits;
// smaller ones round into the half format's last subnormal bits).  float32 models: floats.
template <typename T> struct Operand { typedef T type; };
template <> struct Operand<bf16_t> { typedef f16_t type; };

// Weight-streaming GEMM of the decode step: out[b, n] = sum_k act[b, k] * W[n, k], b < B <= 32.
// HBM-bound.  The matrix's 16-row weight tiles (SwiGLU: gate/up pairs) are shared out evenly over
// n_blocks blocks, at most nw tiles each, over the whole of K (the q|k|v GEMM may also cut K into
// k_split slices for k_split times the blocks: its consumer adds the partial outputs); a block's
// waves split its K range between them, each streaming 1 KiB weight fragments and the matching
// activation fragments (from L2, shared by all the block's tiles) straight into registers, and add
// their sums up through LDS, so nothing of the product goes through memory and no block waits for
// another.
//
// Deferred, centred normalisation: where the GEMM input is Norm(x) = (x - mean) * rstd * gamma + beta,
// the operand holds (x - c) * gamma, written by the producer of x before the row statistics exist,
// with c the row's mean at the previous norm (the embedding uses the row's own mean; RMSNorm: c = 0),
// so that rounding the operand to 11 bits loses nothing to cancellation.  The epilogue applies
// rstd * (acc - (mean - c) * wg[n]) + cb[n]  with wg[n] = sum_k W[n,k] gamma[k] and
// cb[n] = sum_k W[n,k] beta[k] + bias[n], both folded when the weights are uploaded.  mean - c and
// rstd come from the producer's per-tile partial sums (sum (x-c), sum (x-c)^2), added in tile order.
// The first block of shard 0's consumer leaves the new mean in `cen` for the next producer.
struct StreamGemmArgs {
  const void *w;        // weight fragments [row_tiles][k_blocks]
  int row_tiles;        // 16-row tiles (SwiGLU: gate/up tiles interleaved, 2 per 16 outputs)
  int k_blocks;
  int ks;               // waves per block = slices of K (4 or 8)
  int nw;               // weight tiles per block at most (the kernel instance): 1, 2, 3 or 6; SwiGLU: 2 or 6 (whole pairs)
  int n_blocks;         // blocks the tiles (SwiGLU: pairs) are shared out over, evenly: ceil(units / n_blocks) * tiles per unit <= nw
  int u_base, u_rem;    // units / n_blocks and units % n_blocks: block g owns u_base + (g < u_rem) units, in order
  int k_slice;          // k blocks a block covers: ceil(k_blocks / max(1, k_split))
  int B;                // live batch rows
  int N;                // logical output features (for masking)
  const void *act;      // operand fragments [B tiles][k_blocks]
  const void *zero_frag;  // 1 KiB of zeros: the activation fragment of a batch row or a k block that does not exist
  // deferred normalisation (stat_groups > 0)
  const float *stat_in; // [stat_groups][32][4]: two partial (sum, sum of squares) pairs of the rows of x - c per entry
  float *cen;           // [32] or NULL (RMSNorm).  Consumer with publish: cen[b] += mean - c by block 0; EPI_RESID: the centre c
  int publish;
  int stat_groups;
  int norm_dim;         // length of a row of x
  int rms;
  float eps;
  const float *wg;      // [row_tiles * 16] or NULL (RMSNorm)
  const float *cb;      // [row_tiles * 16] folded beta and bias, or the plain bias, or NULL
  // epilogues
  float *out_f32;       // EPI_F32 / EPI_LOGITS: [B][ld_out]
  int ld_out;
  int k_split;          // EPI_F32: S = 2..8 blocks per tile group over a slice of K each, partial outputs at
  size_t part_stride;   //   out_f32 + s * part_stride (floats) for the consumer to add up in order; 0 or 1 = whole K per block
  int split_ok;         //   the most slices the consumer can add (0 or 1: none; set by the plan, the launch rule may then split)
  float split_cost_us;  //   and what adding partial sums costs the consumer (microseconds, for the launch rule)
  const float *x_in;    // EPI_RESID: residual stream before this GEMM, [B][N]
  float *x_out;         // EPI_RESID: after it (may equal x_in)
  void *act_out;        // EPI_ACT / EPI_SWIGLU: activation fragments; EPI_RESID: (x_out - c) * g_out (or NULL)
  int out_k_blocks;
  const float *g_out;   // EPI_RESID: gamma of the norm that follows
  float *stat_out;      // EPI_RESID: [row_tiles / 2][32][4] partial sums of x_out - c, one pair per weight tile (with act_out)
  int act_kind;
  float *am_val;        // EPI_LOGITS: [32][n_blocks] best logit of each block per batch row (written; chosen among by PH_COMMIT)
  int *am_idx;          //             and its vocabulary index (lowest on ties)
  // PH_COMMIT only (the kernel that ends a step; the GEMM kernels do not read these)
  int32_t *next_tokens; // [B] or NULL
  int32_t *lens[8];     // committed lengths to advance (all shards of the group)
  int len_cap[8];       // rows each of those caches holds
  int n_lens;
  int commit_inc;
};
ss_status launch_stream_gemm(int dtype, int epi, const StreamGemmArgs &a, hipStream_t st);
ss_status check_stream_gemm(int dtype, int epi, const StreamGemmArgs &a);  // the shape checks the launcher makes
int stream_gemm_units_per_block(int epi, const StreamGemmArgs &a);  // units (tiles, SwiGLU: pairs) of the largest block
// the activation of a first FFN matrix whose K was cut into slices: adds the partial outputs, writes operand fragments
ss_status launch_act_fixup(int dtype, const StreamGemmArgs &a, hipStream_t st);
ss_status check_act_fixup(int dtype, const StreamGemmArgs &a);
int act_fixup_blocks(const StreamGemmArgs &a);
// wg / cb of a weight matrix in fragment order (gamma NULL: wg is not written)
ss_status launch_fold_norm(int dtype, const void *w, int row_tiles, int k_blocks, const float *gamma, const float *beta,
                           const float *bias, float *wg, float *cb, hipStream_t st);

// Prefill GEMM: out[t, n] = sum_k act[t, k] * W[n, k] over T tokens (multiple of 256), MFMA-bound.
// Norms are deferred as in the decode GEMM, and centred: the residual epilogue of the last shard
// of a group also writes the next GEMM's operand (x - c) * gamma, c = the token's mean at the
// previous norm (0 for RMSNorm), so that rounding the operand to 11 bits costs nothing to
// cancellation, and per token the partial (sum (x-c), sum (x-c)^2) of each 64-feature band a wave
// owns; a small kernel adds the partials up in band order into the token's
// (mean, rstd, mean - c), and the GEMM that consumes the operand applies
// rstd * (acc - (mean - c) * wg[n]) + cb[n].  Tokens past T_live are computed but never stored.
struct TileGemmArgs {
  const void *w;      // weight fragments
  int row_tiles;      // 16-row weight tiles (SwiGLU: 2 per 16 outputs, interleaved)
  int k_blocks;
  const void *act;    // activation fragments [T/16][k_blocks] of the operand type
  const void *act_lo; // or NULL.  The low parts of a two-part operand (act + act_lo carries twice the significant bits):
  int lo_row_begin, lo_row_end;  //   weight row tiles [lo_row_begin, lo_row_end) (multiples of 8) run the reduction a second time over act_lo
  int T;              // tokens (padded to 256)
  int T_live;         // tokens that exist
  int N;
  const float *bias;  // plain bias (mr_in NULL), or NULL
  // deferred normalisation of the input (mr_in != NULL): bias is not read
  const f32x4 *mr_in;     // [T] (mean, rstd, mean - centre of the operand, -) of the rows of x
  const float *wg;    // [row_tiles * 16] or NULL (RMSNorm)
  const float *cb;    // [row_tiles * 16] folded beta and bias, or the plain bias, or NULL
  float *out_f32;     // EPI_F32: [T][ld_out]
  int ld_out;
  // EPI_F32 of a fused q|k|v matrix (k_cache != NULL): the k and v columns go straight into the cache rows of token
  // t = b * kv_S + pos, rounded as the cache stores them; only q goes to out_f32.  With rotary positions (rope != NULL:
  // [position][kv_Dh / 2] (cos, sin)) q and k are rotated first; that needs both halves of a head in one wave, i.e. a
  // block shape for which tile_gemm_rotates() says yes: ask before setting rope
  char *k_cache, *v_cache;  // this layer's planes
  const float2 *rope;
  size_t kv_row_stride, kv_head_stride;  // bytes
  int kv_S, kv_Hs, kv_Dh, kv_dtype;
  float *x_resid;     // EPI_RESID: [T][N]
  const float *g_out; // EPI_RESID: gamma of the norm that follows, or NULL: no operand for a next GEMM
  void *norm_out;     // EPI_RESID with g_out: (x - c) * g_out as fragments [T/16][N / FragK]
  void *norm_out_lo;  // or NULL: what rounding norm_out to the operand type lost, as fragments of the same shape
  const f32x4 *c_in;  // EPI_RESID with g_out: [T], .x = the centre c (the token's mean at the previous norm)
  float2 *stat_out;   // EPI_RESID with g_out: [2 * ceil(row_tiles / 8)][T], one per 64-feature band
  void *act_out;      // EPI_ACT / EPI_SWIGLU: fragments [T/16][out_k_blocks]
  int out_k_blocks;
  int act_kind;
  int n_row_blocks;   // set by the launcher: row blocks of the weight matrix
  int tok_tiles;      // token tiles per wave, 8 or 4: blocks of 256 or 128 tokens (anything else: the launcher chooses both)
  int wave_row_tiles; // weight row tiles per wave, 4 or 8: blocks of 128 or 256 rows (256 only with 256 tokens)
};
ss_status launch_tile_gemm(int dtype, int epi, TileGemmArgs a, hipStream_t st);
// whether the block shape that launch_tile_gemm would take for `a` (without cache arguments) can rotate q and k in its epilogue
bool tile_gemm_rotates(int dtype, const TileGemmArgs &a, int head_dim);
// mr[t] <- (mean, rstd, mean - c, 0) from `groups` partial (sum (x-c), sum (x-c)^2) pairs laid out
// [groups][T], with c = mr[t].x on entry
ss_status launch_row_stats(const float2 *part, int groups, int T, int norm_dim, int rms, float eps, f32x4 *mr,
                           hipStream_t st);

// Decode attention over the committed cache (plus the new token), sequence-split.
struct DecodeAttnArgs {
  const float *qkv;     // [B][3*Hs*Dh] float32: q | k | v of the new token, biases applied
  int qkv_parts;        // partial sums of that shape to add up in order (the GEMM cut K into slices), qkv_stride floats apart; 0 or 1: none
  size_t qkv_stride;
  char *k_cache, *v_cache;   // this layer's planes: [Bmax][Hs][Smax][Dh]
  size_t row_stride, head_stride;  // bytes
  const int32_t *lens;  // committed lengths (device)
  const float2 *rope;   // [Smax][Dh/2] or NULL
  float *part;          // [B*Hs][splits][Dh+4]
  int *counters;        // [B*Hs]
  void *o_out;          // operand fragments [nb][Hs*Dh / FragK]
  int B, Hs, Dh, Smax;
  int kv_dtype;         // cache element type (SS_DTYPE_*)
  int rows_per_block, splits;
  int waves;            // per block: 4, or 16 when one block takes a whole (row, head)
  // norm_dim > 0: qkv holds RAW products (the q|k|v GEMM left out the deferred normalisation and the bias, so that
  // its blocks read no row sums), and every block here applies rstd * (sum - (mean - c) * wg[n]) + cb[n] to the
  // elements it stages, from the producer's partial row sums (as StreamGemmArgs: stat_in, stat_groups, norm_dim,
  // rms, eps, wg, cb over the q|k|v columns); with publish, the block of head 0 (first split) leaves the new mean in cen
  const float *stat_in;
  int stat_groups, norm_dim, rms;
  float eps;
  const float *wg, *cb;
  float *cen;
  int publish;
};
ss_status launch_decode_attn(int dtype, const DecodeAttnArgs &a, hipStream_t st);
ss_status check_decode_attn(const DecodeAttnArgs &a);

// One phase of the decode step = one kernel launch.
enum PhaseKind { PH_EMBED = 0, PH_QKV = 1, PH_ATTN = 2, PH_RESID = 3, PH_FFN_UP = 4, PH_LM_HEAD = 5, PH_COMMIT = 6,
                 PH_FFN_ACT = 7 /* the activation of a first FFN matrix whose K was cut into slices */ };
struct EmbedArgs {
  const float *hidden;    // [rows][d] float32: the previous pipeline stage's output, in place of a token lookup; or NULL
  const int32_t *tokens;  // [rows]
  const void *wte, *wpe;  // [V][d], [max_pos][d] or NULL
  const int32_t *lens;    // decode: position = committed length; NULL: position = row % S
  int S;
  int max_pos;            // rows of the position table (the lookup is clamped to it)
  float *x;               // [rows][d]
  int d, V;
  // operand of the first GEMM, centred on the row's mean c (RMSNorm: c = 0): (x - c) * gamma
  const float *gamma;     // gamma of the first norm
  void *act_out;          // operand fragments [rows / 16][d / FragK]
  void *act_lo_out;       // or NULL: what rounding act_out to the operand type lost, as fragments of the same shape
  int rms;
  // decode step: the row's centred sums and its centre
  float *stat_out;        // [32][4] (sum (x-c), sum (x-c)^2, 0, 0) per row
  float *cen_out;         // [32]
  // initial phase: pstat_out[row] = (sum (x-c), sum (x-c)^2), mr_out[row].x = c
  float2 *pstat_out;      // [rows]
  f32x4 *mr_out;          // [rows]
};

struct Phase {
  int kind;      // PhaseKind; also the timing class
  int gx, gy;    // blocks: (rows, 1), (tile pairs, 1) or (batch*heads, splits)
  int shard;     // index of the shard in the group that owns the phase's scratch
  int epi;       // PH_FFN_UP: the GEMM's epilogue (activation, gate/up pair, or float partial outputs of K slices)
  EmbedArgs e;
  StreamGemmArgs g;   // PH_COMMIT uses B, lens, n_lens, commit_inc and, after an LM head, am_val, am_idx, n_blocks, next_tokens
  DecodeAttnArgs at;
};

// Prefill: rotate q, k; write K/V rows [0, S) of every sequence; then causal attention.
struct PrefillAttnArgs {
  float *qkv;           // [T][3*Hs*Dh] float32 (q rotated in place)
  char *k_cache, *v_cache;
  size_t row_stride, head_stride;
  const float2 *rope;
  void *o_out;          // fragments [T/16][Hs*Dh / FragK] of the operand type (halves for bf16 models)
  int B, S, Hs, Dh, Smax;
  int kv_dtype;
  void *vt;             // half-precision cache: scratch for the transposed values [B*Hs][Dh][s_pad]
  int s_pad;            // S rounded up to 64
};
ss_status launch_prefill_kv_write(int dtype, const PrefillAttnArgs &a, hipStream_t st);
ss_status launch_prefill_attn(int dtype, const PrefillAttnArgs &a, hipStream_t st);

}  // namespace ss
