/*
 * spotshard - one GPU's tensor-parallel share of KV-cached generative decoding,
 * and the KV-cache head re-partition that stateful recovery and dynamic
 * re-parallelization need (after SpotServe, arXiv 2311.15566).
 *
 * C ABI.  Every pointer argument says "host" or "device".  The caller owns all
 * device memory and the HIP stream; the library never allocates device memory.
 * ss_prefill, ss_decode_step, their ss_stage_ forms, ss_kv_repack and ss_shard_reset
 * enqueue work on the given stream and return; outputs are valid after the stream
 * has been synchronized.  The calls that say so below synchronize the stream
 * themselves (creation, ss_committed_len, export / import).  A shard
 * is not thread-safe.  Every call returns
 * an ss_status; argument and state errors are found on the host before anything
 * is launched, and leave committed lengths and committed cache rows untouched.
 * ss_last_error() gives the text of the calling thread's last failure.
 *
 * Tensor conventions (host weights): matrices are row-major, "y = x @ W", in the
 * model's dtype (float32, or bfloat16 bit patterns in uint16); vectors (biases,
 * norm gain/shift) are float32.
 */
#ifndef SPOTSHARD_H
#define SPOTSHARD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ss_shard ss_shard; /* opaque; small host object */

typedef enum {
  SS_OK = 0,
  SS_EINVAL = 1, /* bad argument */
  SS_ENOMEM = 2, /* device_bytes too small / host allocation failed */
  SS_ESTATE = 3, /* cache full, lengths disagree, row not empty, ... */
  SS_EHIP = 4,   /* a HIP call failed; text in ss_last_error() */
  SS_EINTR = 5   /* step stopped by the interruption hook; nothing committed */
} ss_status;

enum { SS_NORM_LAYERNORM = 0, SS_NORM_RMSNORM = 1 };
enum { SS_ACT_GELU_TANH = 0, SS_ACT_RELU = 1, SS_ACT_SWIGLU = 2 };
enum { SS_POS_LEARNED = 0, SS_POS_ROPE = 1 };
enum { SS_DTYPE_F32 = 0, SS_DTYPE_BF16 = 1, SS_DTYPE_F16 = 2 };

/* The full model (Section 2.1: a stack of identical Transformer layers, each
 * multi-head attention + FFN).  Pre-norm blocks, final norm, greedy LM head. */
typedef struct {
  int32_t n_layers, d_model, n_heads, head_dim, ffn, vocab;
  int32_t max_pos;  /* rows of the learned position table (0 for RoPE) */
  int32_t norm, act, pos, has_bias;
  int32_t dtype;    /* element type of the weights handed over: SS_DTYPE_F32 or SS_DTYPE_BF16.  A bf16 model is
                       computed with IEEE-half matrix-core operands and float32 accumulation: activations are
                       rounded to halves (11 significant bits; bf16's 8 miss the logits bar), and the weight
                       matrices are held as halves (exact for magnitudes from 2^-17 up, saturating at +-65504). */
  int32_t kv_dtype; /* cache element: SS_DTYPE_F32 for an f32 model; SS_DTYPE_F16 or SS_DTYPE_BF16
                       (both 2 bytes) for a bf16 model.  Half keeps 3 more mantissa bits: bf16 keys
                       alone cost ~4e-3 relative logits error at the OPT-66B shape, half ~6e-4;
                       values saturate at +-65504. */
  float norm_eps, rope_theta;
} ss_model_desc;

/* What one pipeline-stage-shard position (d, p, m) of a parallel configuration
 * holds (Section 3.3): consecutive layers (the stage), whole heads and FFN
 * columns (the tensor-parallel shard, Section 2.2).  Half-open intervals in the
 * full model's index space. */
typedef struct {
  int32_t layer_lo, layer_hi, head_lo, head_hi, ffn_lo, ffn_hi;
} ss_slice;

/* Host pointers to one layer's PARENT tensors.  With Hp/Fp the parent's head and
 * FFN counts and Dh = head_dim:
 *   wq wk wv [d, Hp*Dh]   bq bk bv [Hp*Dh]      wo [Hp*Dh, d]   bo [d]
 *   w1 [d, Fp]  b1 [Fp]   (GELU / ReLU)          wg wu [d, Fp]   (SwiGLU)
 *   w2 [Fp, d]  b2 [d]    ln1_g ln1_b ln2_g ln2_b [d]
 * Pointers of absent tensors (biases when has_bias = 0, norm shifts for RMSNorm)
 * are NULL. */
typedef struct {
  const void *ln1_g, *ln1_b, *wq, *wk, *wv, *bq, *bk, *bv, *wo, *bo;
  const void *ln2_g, *ln2_b, *w1, *b1, *wg, *wu, *w2, *b2;
} ss_layer_weights;

/* Host pointers to the model context a shard is cut from.  `slice` says which
 * part of the full model the tensors cover (a parent may itself be a shard).
 *   wte [vocab, d]   wpe [max_pos, d] or NULL   lm_head [vocab, d] (may equal wte;
 *   logits = xf @ lm_head^T)   lnf_g lnf_b [d]
 *   layers[i] is layer slice.layer_lo + i. */
typedef struct {
  ss_slice slice;
  const void *wte, *wpe, *lm_head, *lnf_g, *lnf_b;
  const ss_layer_weights *layers;
} ss_weights;

/* A position's two kinds of context (Section 3.1: the context daemon keeps the model context,
 * i.e. the parameters, and the cache context, i.e. the keys and values, in device memory; Section 5:
 * the engine takes its tensors from the daemon instead of allocating them).
 * Device bytes a shard needs for its model context (weights, re-laid out for the
 * matrix cores), its cache context (K and V of every layer, max_batch x max_seq
 * rows) and its workspace.  0 on invalid arguments. */
size_t ss_shard_device_bytes(const ss_model_desc *desc, const ss_slice *slice,
                             int32_t max_batch, int32_t max_seq);

/* Create the shard for `slice`: copies that slice of the parent's tensors (host)
 * into `device_mem` (device, 256-byte aligned, at least ss_shard_device_bytes();
 * owned by the caller and must outlive the shard) on `hip_stream`, and
 * synchronizes the stream before returning, so the host tensors may be released.
 * All committed lengths start at 0.  SS_EINVAL if the slice is not inside the
 * parent's slice or a shape is unsupported; SS_ENOMEM if device_bytes is short. */
ss_status ss_shard_create(const ss_model_desc *desc, const ss_slice *slice,
                          const ss_weights *parent, int32_t max_batch, int32_t max_seq,
                          void *device_mem, size_t device_bytes, void *hip_stream,
                          ss_shard **out);

/* Model-context migration on one device (Section 3.3: the device mapper maximises the model
 * parameters a device can re-use in its new position): a shard for `slice` whose model context is
 * copied, device to device, out of resident shards of the same model instead of being uploaded
 * again.  Every (layer, head) and (layer, FFN column) of `slice` must be held by one of
 * `sources` (in any order; FFN columns shared with a source in multiples of 64), else SS_EINVAL.
 * The result is bit-identical to what ss_shard_create builds from the host tensors; its cache is
 * empty.  The sources are only read.  Synchronizes the stream.  bytes_copied (host, may be NULL)
 * receives the bytes of model context moved. */
ss_status ss_shard_create_from_resident(const ss_model_desc *desc, const ss_slice *slice,
                                        ss_shard *const *sources, int32_t n_sources, int32_t max_batch,
                                        int32_t max_seq, void *device_mem, size_t device_bytes,
                                        void *hip_stream, ss_shard **out, uint64_t *bytes_copied);

/* Bytes at the start of a shard's device_mem that hold its model context (everything before the
 * cache): what a byte-for-byte comparison of two shards' model context covers. */
size_t ss_shard_model_context_bytes(const ss_shard *shard);

/* A position whose context has been migrated away gives its memory back (Section 3.4: migrated
 * context is released as the plan proceeds): frees the host object and its captured graphs; the
 * device memory is the caller's. */
ss_status ss_shard_destroy(ss_shard *shard);

/* Drop the cache context: every committed length back to 0 (Section 4.2: a
 * position that lost its cache falls back to recomputing it). */
ss_status ss_shard_reset(ss_shard *shard, void *hip_stream);

/* Initial phase (Section 2.1, Eq. (1) first term): all S_in prompt tokens of B
 * sequences in parallel under the causal mask; fills cache rows [0, S_in) and
 * commits n[b] = S_in; logits of the last position and the greedy first output
 * token.  `group`: 1..8 co-resident shards (host array of handles) holding the
 * same layers with disjoint head and FFN intervals; their partial attention and
 * FFN outputs are summed where a tensor-parallel group would All-Reduce
 * (Section 2.2); embedding, norms, row-parallel biases and LM head come from
 * group[0].  tokens: device int32 [B, S_in].  logits: device float32 [B, vocab]
 * or NULL.  next_tokens: device int32 [B] or NULL.  SS_ESTATE unless rows [0,B)
 * are empty in every shard; SS_EINVAL if B > max_batch or S_in > max_seq. */
ss_status ss_prefill(ss_shard *const *group, int32_t n_group, const int32_t *tokens,
                     int32_t B, int32_t S_in, float *logits, int32_t *next_tokens,
                     void *hip_stream);

/* One incremental decoding iteration (Section 2.1, Eq. (2)): row b consumes
 * tokens_in[b] at position n[b], its key/value become cache row n[b], it attends
 * over rows 0..n[b]; logits and greedy next token (lowest index on ties) come
 * out; then, as the last stream-ordered action, n[b] <- n[b] + 1 (token-level
 * commit, Section 4.1).  Row n[b] is not part of the committed state before that.
 * tokens_in: device int32 [B]; logits: device float32 [B, vocab] or NULL;
 * next_tokens: device int32 [B] or NULL (may alias tokens_in).
 * SS_ESTATE if a row's cache is full or the group's lengths disagree.
 * The step's kernels are captured into a HIP graph the first time a combination of (group, batch size, tokens_in,
 * logits, next_tokens, stream) is seen, and replayed from then on; the group's first shard keeps up to 16 such graphs
 * (a caller that hands in other buffers at every step pays the capture every time: keep the buffers).  On the NULL
 * stream, or on a stream the caller is capturing, the kernels are launched one by one. */
ss_status ss_decode_step(ss_shard *const *group, int32_t n_group, const int32_t *tokens_in,
                         int32_t B, float *logits, int32_t *next_tokens, void *hip_stream);

/* ss_decode_step for callers that cannot allocate device memory or let the library do so (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * iteration with the same kernels and the same bits, but the step's scratch (residual rows,
 * operand fragments, row sums, q|k|v, attention partials and counters, LM-head candidates) lives
 * in a static device array of ss_static_scratch_bytes() = 32 MiB that every device the library
 * runs on holds until the process ends, the kernels are launched one by one (no graph is
 * instantiated), and no hipMalloc / hipFree or allocating library routine is called.  The caller
 * still passes the inputs and outputs; the shards' caches and weights stay where they are.
 * SS_ENOMEM if a step of this group needs more scratch than the array holds (nothing is launched);
 * otherwise the errors of ss_decode_step.  Every call on a device shares that device's array:
 * calls that overlap on one device (two streams, two threads) race; calls in stream order are fine. */
size_t ss_static_scratch_bytes(void);
ss_status ss_decode_step_static(ss_shard *const *group, int32_t n_group, const int32_t *tokens_in,
                                int32_t B, float *logits, int32_t *next_tokens, void *hip_stream);

/* The same two calls for a shard that is one STAGE of a pipeline (Section 2.2, inter-operator
 * parallelism: consecutive layers grouped into stages, each fed by the one before).  Exactly
 * one of tokens / hidden_in is given: tokens for the model's first stage, hidden_in (device
 * float32, [B * S_in, d_model] for the initial phase, [B, d_model] for a step: the previous
 * stage's hidden_out) for a later one, which then skips the embedding.  With hidden_out (device
 * float32, same shapes) the shard is not the last stage: the residual stream after its layers
 * goes there, no final norm or LM head runs (logits and next_tokens must be NULL) and the
 * commit is the step's last kernel all the same.  hidden_out = NULL: final norm, LM head,
 * greedy token as in ss_prefill / ss_decode_step, which are these calls with tokens only.
 * SS_EINVAL if both or neither of tokens / hidden_in are given. */
ss_status ss_stage_prefill(ss_shard *const *group, int32_t n_group, const int32_t *tokens,
                           const float *hidden_in, int32_t B, int32_t S_in, float *hidden_out,
                           float *logits, int32_t *next_tokens, void *hip_stream);
ss_status ss_stage_decode_step(ss_shard *const *group, int32_t n_group, const int32_t *tokens_in,
                               const float *hidden_in, int32_t B, float *hidden_out, float *logits,
                               int32_t *next_tokens, void *hip_stream);

/* The progress a request has committed (Section 4.1: progress is committed per token, so an
 * interrupted request resumes from its last committed token).  Committed lengths as the device
 * holds them: synchronizes the stream, copies n[0..max_batch) to out_host (host int32 [max_batch]). */
ss_status ss_committed_len(const ss_shard *shard, int32_t *out_host, void *hip_stream);

/* Cache-context migration on one device (Section 3.3: a device re-uses the
 * intersection of the context it holds with the context its new position needs).
 * For every layer in both layer intervals, K and V, every destination row b' with
 * b = batch_map[b'] >= 0 (host int32 [dst max_batch]; -1 = leave the row alone;
 * dropping rows is the cache-discard case), every head in both head intervals:
 * copies committed rows [0, n_src[b]) bit for bit into dst's layout and sets
 * n_dst[b'] = n_src[b].  src is not modified; dst rows >= n, unmapped rows and heads
 * outside the intersection are left as they were.  A merge calls this once per
 * source; SS_ESTATE if a later source disagrees with the length dst already holds
 * for a row that an earlier source of the same merge filled (pass first_source = 0
 * for those calls), or if n_src[b] exceeds dst's max_seq.  SS_EINVAL if dtype or
 * head_dim differ, a source row is mapped twice, or src == dst.
 * bytes_moved (host, may be NULL) receives the payload bytes copied. */
ss_status ss_kv_repack(ss_shard *dst, const ss_shard *src, const int32_t *batch_map,
                       int32_t first_source, uint64_t *bytes_moved, void *hip_stream);

/* The cache context as what migration moves between devices (Section 3.4: cache context is
 * migrated first; Section 4.1: a request resumes on the new configuration from its committed
 * keys and values without recomputing them): committed cache rows to / from host memory in the exchange order
 * [layer][K|V][b][head][j < n[b]][Dh], densely packed, in the cache dtype.
 * ss_kv_export_bytes gives the size for the current lengths.  Import sets the
 * lengths to lens (host int32 [max_batch]) and expects exactly that many bytes.
 * Both synchronize the stream. */
size_t ss_kv_export_bytes(const ss_shard *shard);
ss_status ss_kv_export(const ss_shard *shard, void *host_dst, size_t bytes, void *hip_stream);
ss_status ss_kv_import(ss_shard *shard, const void *host_src, const int32_t *lens,
                       size_t bytes, void *hip_stream);

/* Geometry of the shard, for callers that size buffers: out[0..5] = layers, heads,
 * ffn columns, max_batch, max_seq, bytes per cache element. */
ss_status ss_shard_geometry(const ss_shard *shard, int32_t out[6]);

/* Text of the calling thread's last failure.  Plumbing of this boundary (the paper defines no
 * error interface; Section 4.2 only says what the system falls back to when a step or a migration
 * cannot go ahead: the caller needs to know which).  Thread-local, never NULL. */
const char *ss_last_error(void);
const char *ss_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPOTSHARD_H */
