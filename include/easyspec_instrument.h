/*
 * easyspec_instrument.h — measurement and test hooks of the EasySpec draft library (same shared
 * library as easyspec.h).  None of them is part of the method (Alg. 2 / Sec. 3.2 / Alg. 3 of arXiv
 * 2502.02493): they time the kernels, probe the device's streaming rate, evaluate the kernels' index
 * arithmetic on the host, and poison workspaces, for the benchmark and the tests.  Conventions as in
 * easyspec.h.
 */
#ifndef EASYSPEC_INSTRUMENT_H
#define EASYSPEC_INSTRUMENT_H

#include "easyspec.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Fill every workspace a forward pass uses between its kernels (residual stream, norm operands and partial
 * sums, queries, attention output and split-KV partials, parked Attnoutputs, MLP activations, argmax
 * candidates) with NaN bit patterns, on the context's stream.  Weights, the KV cache and the lengths are not
 * touched.  A forward pass writes each of these before it reads it, so a call between two passes must
 * change no result bit: for tests of exactly that (a kernel that read a workspace entry no earlier kernel
 * of the same pass wrote would turn its output into NaN). */
int easyspec_poison_workspaces(easyspec_ctx *ctx);

/* Streaming-read probe for roofline reports: reads `bytes` (a positive multiple of 16) of the
 * caller's device buffer once, with the loads the weight stream uses (16-byte, non-temporal,
 * 8 in flight per lane), on hip_stream (NULL = the null stream).  The caller times it; the rate
 * is what a kernel that only reads can reach on this device, against which the share of the
 * nominal 8 TB/s can be judged.  sink: dev, easyspec_stream_read_sink_floats() floats, receives
 * checksums so that the reads cannot be dropped.  EASYSPEC_EINVAL for NULL or a bad size. */
int easyspec_stream_read(const void *buf, int64_t bytes, float *sink, void *hip_stream);
int32_t easyspec_stream_read_sink_floats(void);

/* How a decode-attention launch over n_layers_in_set layers would cut the contexts of n_cols
 * columns among workgroups and waves (the split-KV cut of the vector-ALU attention kernel): host
 * arithmetic only, evaluated with the kernels' own index functions, no device needed.  For tests
 * of that arithmetic (every slot of every column must fall to exactly one wave) and for tuning.
 *   ctx_lens  host [n_cols]  slots column i attends to (1 .. max_ctx), n_cols 1 .. 16
 *   n_chunks  host [n_cols]  receives the chunks of column i (1 .. EASYSPEC_MAX_CHUNKS)
 *   ranges    host [n_cols][EASYSPEC_MAX_CHUNKS][8][2] or NULL: receives the slots [from, to) of
 *             wave w of chunk c of column i; (0, 0) beyond the column's chunks or the launch's waves
 * Returns the waves per workgroup of the launch (4 or 8), or a negative error code. */
#define EASYSPEC_MAX_CHUNKS 64
int easyspec_attention_cut(const easyspec_config *cfg, const int32_t *ctx_lens, int32_t n_cols, int32_t n_layers_in_set,
                           int32_t *n_chunks, int32_t *ranges);

/* Host model of the weight stream of one launch of a weight-streaming kernel class (EASYSPEC_OP_QKV,
 * _OPROJ, _GATEUP, _DOWN, _HEAD) with n_cols token columns over n_layers_in_set layers (full_layer != 0:
 * the launch shapes of the full-layer-parallel mode): every workgroup, wave and lane of the grid computes,
 * with the kernels' own index functions and the launch wrappers' own choice of grid, waves and tile
 * heights, each 16-byte piece of weights and each activation fragment it would load.  Host arithmetic
 * only, no device needed: for tests that no launch shape reads outside its packed matrices or operand
 * slot, skips a k-tile or reads one twice.  report (host, EASYSPEC_WALK_FIELDS entries):
 *   [0] grid, [1] waves per workgroup, [2] units (row tiles) per workgroup, [3] rows per tile,
 *   [4] activation fragments per k-tile,
 *   [5] highest piece index read, [6] pieces the launch's layers hold, [7] reads outside them,
 *   [8] highest activation element read, [9] elements of an operand slot, [10] reads outside it,
 *   [11] k-tiles of the launch, [12] never read, [13] read more than once, [14] deliberate re-reads of a
 *   missing last unit (results dropped), [15] fragment pieces that no lane takes. */
#define EASYSPEC_WALK_FIELDS 16
int easyspec_weight_walk(const easyspec_config *cfg, int32_t op, int32_t n_cols, int32_t n_layers_in_set, int32_t full_layer,
                         int64_t *report);

/* Host model of how the vector attention kernel, where it takes its scores from the matrix cores (bf16
 * caches, head_dim 128, 4 to 8 query heads per KV head), passes a batch of n_loads x 4 K rows (n_loads = 2:
 * a short step, 8: a full batch) through a wave's LDS into MFMA A fragments, evaluated with the kernel's own
 * index functions for all 64 lanes.  Host arithmetic only.  report (host, EASYSPEC_STAGE_FIELDS entries):
 *   [0] 16-byte pieces stored, [1] distinct places they take, [2] highest place + 1, [3] places a wave owns,
 *   [4] fragment pieces fetched from rows of the batch, [5] of those, fetches that do not return the piece
 *   (slot, 32-element k-tile, k-group) the MFMA operand needs there, [6] fetches from rows the batch does not
 *   have (their scores are never used), [7] (lane, load) pairs whose score would come out in another lane or
 *   element than the one that holds the slot's V row, [8] pairs of lanes of one quarter-wave that meet in one
 *   16-byte bank group, stores and fetches together. */
#define EASYSPEC_STAGE_FIELDS 9
int easyspec_attention_stage_walk(int32_t n_loads, int64_t *report);

/* Per-kernel timing for roofline reports.  Between profile_begin and profile_end every kernel
 * launch of the class `op` made by draft steps and calibrations carries a start and a stop HIP
 * event bound to its own dispatch (at most max_launches launches; later ones run untimed), so a
 * pair's elapsed time is that kernel's begin-to-end time.  With EASYSPEC_OP_ALL every launch of
 * the forward pass is timed, which is what a kernel trace does and gives the figures that compare
 * with one (a timed kernel that follows an untimed one also counts part of its predecessor's tail).
 * profile_end synchronises the stream and returns the number of timed launches, the sum of their
 * durations in milliseconds and, where launch_ms / launch_op are not NULL (host, max_launches
 * entries each), every launch's duration and kernel class in launch order (the embedding gather
 * reports EASYSPEC_OP_ALL).  A class with two kernels per use (attention: partial + merge; head:
 * logits + argmax) counts each kernel as a launch.  Not meant to stay on in production. */
#define EASYSPEC_OP_QKV 0    /* stacked QKV projection + rotary + cache write */
#define EASYSPEC_OP_ATTN 1   /* split-KV decode attention (partial + merge kernels together) */
#define EASYSPEC_OP_OPROJ 2  /* stacked O projection */
#define EASYSPEC_OP_GATEUP 3 /* gate/up projection + SiLU*up */
#define EASYSPEC_OP_DOWN 4   /* down projection + residual */
#define EASYSPEC_OP_HEAD 5   /* LM head + argmax (both kernels together) */
#define EASYSPEC_OP_ALL 6    /* every kernel of the forward pass, the embedding gather included */
int easyspec_profile_begin(easyspec_ctx *ctx, int32_t op, int32_t max_launches);
int easyspec_profile_end(easyspec_ctx *ctx, int32_t *n_launches, float *total_ms, float *launch_ms, int32_t *launch_op);

#ifdef __cplusplus
}
#endif
#endif /* EASYSPEC_INSTRUMENT_H */
