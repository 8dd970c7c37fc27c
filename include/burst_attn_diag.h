/*
 * libburstattn -- diagnostics.  Not part of the attention path: host-side views of the kernels' tile
 * logic for tests, and a matrix-core ceiling probe for benchmarks.  Conventions as in burst_attn.h.
 */
#ifndef BURST_ATTN_DIAG_H
#define BURST_ATTN_DIAG_H

#include "burst_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Host diagnostics of the tile-level mask logic, running the very code the kernels compile (no GPU
 * involved), so that tests can hold it against a brute-force visibility matrix.
 *
 * burst_attn_tile_class: class of the block of query rows [q0, q1) against key rows [k0, k1):
 * 0 = no pair visible (the kernels skip the tile), 1 = every pair visible (no per-element predicate),
 * 2 = mixed.  method 0: the direct position-range test; 1: the per-segment row thresholds the
 * key-stationary kernel derives once for a fixed key range; 2: the same for a fixed query range
 * (query-stationary kernels).  All three must agree.  Negative burst_status_t on a bad argument.
 *
 * burst_attn_visible_tile_runs: the tiles of `tile_rows` rows along the query axis (query_axis != 0;
 * tile_rows 64 or 256) or the key axis (tile_rows 64 or 128) that can hold a pair visible to rows
 * [r0, r1) of the other axis, as at most two runs: out = {start0, len0, start1, len1} in tiles. */
int burst_attn_tile_class(const burst_mask_t* mask, int64_t q0, int64_t q1, int64_t k0, int64_t k1, int32_t method);
int burst_attn_visible_tile_runs(const burst_mask_t* mask, int32_t query_axis, int32_t tile_rows, int64_t r0, int64_t r1,
                                 int32_t out_start_len[4]);

/* Diagnostic, not part of the attention path: enqueues `iterations` x 4 independent bf16 32x32x16
 * MFMAs per wave on every SIMD (512 work-groups of 256 threads) with constant (0) or pseudo-random
 * (1) register operands, and stores the flop count of the launch in *flops_out (host, optional).
 * Timed by the caller with events, it gives the matrix-core ceiling of the chip as it is clocked under
 * that load: dense attention tiles are bounded by the random-operand figure.  sink: optional device
 * pointer to 4 bytes (never written in practice).  iterations in [1, 2^24]. */
int burst_attn_mfma_probe(int32_t random_operands, int32_t iterations, float* sink, int64_t* flops_out,
                          void* hip_stream);

/* The step kernels cut a streamed axis (keys for the forward kernel when it only updates the running state,
 * and for dQ; queries for dK / dV) that is longer than twice `rows` into ranges of about `rows` rows, one
 * launch per range (an L2-locality measure; default 32768).  Tests lower it to drive the chunked path at sizes
 * the oracle can check exhaustively.  Process-wide; values below 256 are raised to 256.  Returns the value now
 * in force. */
int burst_attn_set_chunk_rows(int32_t rows);

/* Host view of that plan (no GPU involved): the ranges of local rows the query axis (query_axis != 0: the
 * dK/dV kernel's launches) or the key axis (the dQ kernel's and the forward kernel's) of a step with this mask is cut into.  Returns
 * the number of ranges (negative burst_status_t on a bad mask) and fills, for the first max_ranges of them,
 * out[7 i ..] = {first row, end row, pieces, rows per piece, position of the first row, position period of
 * the pieces, byte offset of the range's block mask from the step's} -- the chunk the range's launch
 * describes to the kernel.  One range means one launch with the step's own mask. */
int burst_attn_chunk_plan(const burst_mask_t* mask, int32_t query_axis, int32_t max_ranges, int64_t* out);

#ifdef __cplusplus
}
#endif
#endif /* BURST_ATTN_DIAG_H */
