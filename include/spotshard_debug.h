/*
 * spotshard - test hooks and measurement aids.  Not part of the serving boundary (spotshard.h):
 * the tests use them to force code paths and launch shapes, bench.py to time kernel classes.
 */
#ifndef SPOTSHARD_DEBUG_H
#define SPOTSHARD_DEBUG_H

#include "spotshard.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Test hook for "a request can be interrupted at any iteration" (Section 4.1):
 * with layer >= 0 the next decode steps stop after that layer (index within the
 * shard) and return SS_EINTR without committing.  -1 switches it off. */
ss_status ss_debug_interrupt_after_layer(ss_shard *shard, int32_t layer);

/* How ss_decode_step is launched.  1 (default): replay of a captured HIP graph of the step's
 * kernels; 0: the kernels one by one.  Both give the same bits. */
ss_status ss_set_graph_launch(ss_shard *shard, int32_t enabled);

/* Test aid, process-wide: force the launch shape of the decode GEMMs built from now on (a shard's
 * captured graphs are keyed by the forced shape, so the change takes effect at once): weight tiles per
 * block at most (1, 2, 3 or 6; where a GEMM has no such kernel instance the nearest one; 0 = the
 * library's choice) and the slices the q|k|v GEMM cuts K into (1..8; 0 = the library's choice; with more
 * than 16 batch rows the first FFN matrix of a model without gate is cut the same way and its activation
 * becomes a kernel of its own; other GEMMs never cut K).  The library chooses per shape by a cost rule.
 * The tiles per block never change a bit of the result; the number of K slices changes the order of the
 * sums. */
ss_status ss_debug_force_gemm_shape(int32_t tiles_per_block, int32_t k_slices);

/* Test aid, process-wide: force the block of the initial phase's tiled GEMMs (the initial
 * phase over all prompt tokens: the first term of Eq. (1) and Eq. (2)): 128 weight rows x 128 tokens, 128 x 256 or
 * 256 x 256; 0 x 0 = the library's choice, which goes by the size of the output (a GEMM whose two-part operand
 * does not cover whole 256-row blocks keeps 128 rows).  All give the same bits.  SS_EINVAL for any other pair. */
ss_status ss_debug_force_prefill_block(int32_t rows_per_block, int32_t tokens_per_block);

/* Measurement aid for the roofline of the initial phase's GEMM (the first term of Eq. (1); matrix-core bound): what the
 * matrix cores sustain on the caller's operand data.  One block of four waves per compute unit runs `iters` times 64
 * half-precision 16x16x32 products per wave on fragments taken from operands_dev (device memory, operand_bytes of it, 1 MiB to
 * 4 GiB, read only; any bit pattern), optionally with the LDS reads (16 KiB per 64 products and wave) and the direct-to-LDS
 * loads (8 KiB, from operands_dev) that the GEMM's 256-row block issues per stage.  Returns the rate in TFLOP/s, the
 * cycles per 64 products and the clock (cycle counter over event time).  The clock under matrix-core load depends on
 * the operand data: compare constant with random operands.  Allocates and frees a few KiB of device memory and
 * synchronizes on its own events; SS_EINVAL for bad arguments, SS_EHIP if the runtime fails. */
ss_status ss_debug_matrix_core_probe(const void *operands_dev, uint64_t operand_bytes, int32_t lds_reads, int32_t loads,
                                     int32_t iters, double *tflops, double *cycles_per_64, double *ghz, void *hip_stream);

/* Measurement aid: per-kernel-class timing of decode steps.  While enabled on group[0],
 * ss_decode_step launches kernel by kernel (no graph replay) and every launch records its own
 * begin and end on a pair of HIP events of the step's stream (the dispatch's timestamps).
 * ss_kernel_timing_read synchronizes the stream, returns the milliseconds and launch counts
 * accumulated per class since the last read (host arrays of 8) and clears them.  Classes:
 * 0 embedding, 1 QKV GEMM, 2 decode attention, 3 out-projection and second-FFN GEMM (the
 * residual epilogue), 4 first-FFN GEMM, 5 LM head, 6 the kernel that ends a step (greedy choice among
 * the LM head's per-block candidates, if there is an LM head, then the token-level commit). */
ss_status ss_kernel_timing(ss_shard *shard, int32_t enabled);
ss_status ss_kernel_timing_read(ss_shard *shard, double ms[8], int64_t count[8], void *hip_stream);

/* Host-only check aid (no device memory is touched): the phase table one decode step would use
 * for a shard of this shape placed at device address fake_base.  See the implementation for
 * the record layout; used by the CPU tests that bound-check every buffer a phase addresses. */
int32_t ss_debug_plan(const ss_model_desc *desc, const ss_slice *slice, int32_t max_batch, int32_t max_seq,
                      int32_t B, uint64_t fake_base, void *out_phases, int32_t max_phases, uint64_t *out_total,
                      uint64_t *out_sizeof_phase);

#ifdef __cplusplus
}
#endif
#endif /* SPOTSHARD_DEBUG_H */
