/*
 * spotshard - host-side planning for a change of parallel configuration (after SpotServe,
 * arXiv 2311.15566): how much context two positions share, which device should take which
 * position, in what order the layers' context moves, which requests keep their cache, how
 * many decoding iterations fit into a grace period, and what an inference costs.  Plain host arithmetic on small inputs: no
 * GPU, no allocation that outlives a call; every pointer is a host pointer.  Same ss_status and
 * ss_last_error() as spotshard.h.
 */
#ifndef SPOTSHARD_PLAN_H
#define SPOTSHARD_PLAN_H

#include "spotshard.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Size of the intersection of the contexts of two positions (Section 3.3: the edge weight between
 * a device and a position is the amount of model parameters and KV cache it could re-use there).
 * Model context: for every layer in both layer intervals the Q/K/V and output-projection elements
 * of the heads in both head intervals, the FFN elements of the columns in both FFN intervals, the
 * biases that go with them, and the layer's replicated vectors (norm gain/shift, the two
 * row-parallel biases); plus the replicated embedding tables, final norm and LM head (counted once
 * when lm_head_tied).  Cache context: layers x {K, V} x common heads x head_dim x kv_rows, where
 * kv_rows is the sum of the committed lengths of the requests the new position inherits from the
 * old one (0 if it inherits none).  Bytes in the model's weight / cache element sizes (vectors
 * float32). */
ss_status ss_context_overlap(const ss_model_desc *desc, int32_t lm_head_tied, const ss_slice *a, const ss_slice *b,
                             uint64_t kv_rows, uint64_t *model_bytes, uint64_t *cache_bytes);

/* Device mapping (Section 3.3): a maximum-weight perfect matching of n devices to n positions
 * (Kuhn-Munkres), weight[u * n + v] = re-usable bytes when device u takes position v.
 * position_of[u] receives the position of device u, *total the matched weight.  Among equal
 * optima the result is deterministic.  n in [1, 512]. */
ss_status ss_match_devices(int32_t n, const uint64_t *weight, int32_t *position_of, uint64_t *total);

/* Order in which the layers' model context migrates (Algorithm 2, memory-optimised planner).
 * delta[l * n_instances + i] = change of instance i's buffer memory (bytes, signed: receivers
 * grow, senders shrink) when layer l's context migrates.  First the layers in index order whose
 * migration keeps every instance at or below u_max; then, of the layers left out, repeatedly the
 * one whose migration gives the smallest maximum over the instances (lowest index on ties).
 * order receives n_layers layer indices. */
ss_status ss_migration_order(int32_t n_layers, int32_t n_instances, const int64_t *delta, int64_t u_max,
                             int32_t *order);

/* The progressive plan (Algorithm 2, first function): all cache context first, then the layers in
 * `order`; a stage starts as soon as all of its layers have arrived.  stage_of_layer[l] in
 * [0, n_stages).  Writes 1 + n_layers + n_stages entries: kind[k] = 0 migrate cache (arg -1),
 * 1 migrate layer arg[k], 2 start stage arg[k]. */
enum { SS_PLAN_MIGRATE_CACHE = 0, SS_PLAN_MIGRATE_LAYER = 1, SS_PLAN_START_STAGE = 2 };
ss_status ss_progressive_plan(int32_t n_layers, const int32_t *order, const int32_t *stage_of_layer, int32_t n_stages,
                              int32_t *kind, int32_t *arg);

/* Cache discard (Section 3.3, last paragraph): when the new configuration holds fewer concurrent
 * requests, the requests with the most decoding progress keep their cache.  lens[r] = committed
 * length of source row r (0 = empty row, never kept); the `keep` rows with the largest lengths
 * (lowest row on ties) are mapped to destination rows 0, 1, ... in source-row order;
 * batch_map[0 .. n_dst) receives the source row of each destination row or -1: the argument
 * ss_kv_repack takes. */
ss_status ss_rows_to_keep(int32_t n_rows, const int32_t *lens, int32_t keep, int32_t n_dst, int32_t *batch_map);

/* Just-in-time arrangement (Section 4.1).  l_exe[S], S = 0 .. s_out: execution latency of
 * generating S tokens under the current configuration (non-decreasing).  Preemption
 * (acquisition = 0): the largest S with l_exe[S] < t_grace - t_mig.  Acquisition: the smallest S
 * with l_exe[S] >= t_grace (s_out if none).  If t_mig >= l_exe[S] the arrangement would only add
 * latency and 0 is returned (re-route instead). */
int32_t ss_jit_iterations(int32_t acquisition, int32_t s_out, const double *l_exe, double t_grace, double t_mig);

/* Measured cost model (Section 5: a cost model and an offline profiler estimate the inference
 * latency in advance; here the profile is a handful of timings taken on the running shard).
 * t_exe of Eq. (1): the initial phase over s_in tokens per sequence costs
 * pre_base_ms + pre_per_token_ms * s_in, an incremental iteration with n tokens already cached
 * costs dec_base_ms + dec_per_row_ms * n (the weights are streamed once whatever n is, the cache
 * rows once each: both terms are linear).  One line per batch size, fitted by least squares;
 * between two fitted batch sizes the predicted times are interpolated linearly, outside them the
 * nearest one is used. */
enum { SS_COST_MAX_BATCHES = 16 };
typedef struct {
  int32_t batch;    /* sequences in the batch */
  int32_t length;   /* decode sample: tokens already cached; initial-phase sample: s_in */
  double ms;        /* measured time of one iteration (or the mean of several around `length`) */
} ss_cost_sample;
typedef struct {
  int32_t n_batches;
  int32_t batch[SS_COST_MAX_BATCHES];   /* ascending */
  double dec_base_ms[SS_COST_MAX_BATCHES], dec_per_row_ms[SS_COST_MAX_BATCHES];
  double pre_base_ms[SS_COST_MAX_BATCHES], pre_per_token_ms[SS_COST_MAX_BATCHES];
} ss_cost_model;

/* Least-squares lines through the samples of each batch size.  A batch size with samples at one
 * length only gets a constant (decode) or a line through the origin (initial phase); a batch
 * size needs at least one decode sample, without initial-phase samples its two initial-phase
 * coefficients are 0.  At most SS_COST_MAX_BATCHES distinct batch sizes.  Caller owns everything. */
ss_status ss_cost_fit(const ss_cost_sample *decode, int32_t n_decode, const ss_cost_sample *prefill, int32_t n_prefill,
                      ss_cost_model *model);

/* Eq. (1): l_exe[S] = t_exe(s_in) + sum_{i=1..S} t_exe(s_in + i) for S = 0 .. s_out, in ms: the
 * table ss_jit_iterations takes.  The i-th incremental iteration runs with s_in + i - 1 tokens
 * cached.  With dec_per_row_ms = 0 this is Eq. (2). */
ss_status ss_cost_l_exe(const ss_cost_model *model, int32_t batch, int32_t s_in, int32_t s_out, double *l_exe);

#ifdef __cplusplus
}
#endif
#endif /* SPOTSHARD_PLAN_H */
