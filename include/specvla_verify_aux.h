/*
 * libspecvla_verify - measurement and inspection aids.  Nothing here is part of the
 * verification path (include/specvla_verify.h); benchmarks and tests use these calls to look
 * inside it.  Same conventions: plain C, [host] / [device] tags, int status, the caller owns
 * every buffer.
 */
#ifndef SPECVLA_VERIFY_AUX_H
#define SPECVLA_VERIFY_AUX_H

#include "specvla_verify.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Host-only inspection aid for tests: where an intermediate of the last sv_verify_layer call
 * lives inside the workspace.  which = SV_WS_ATTN_OUT: attention output before the output
 * projection, float32 [B*T, nh*d].  which = SV_WS_Q: rotated queries, float32 [B*T, nh*d].
 * which = SV_WS_STATUS: one int32 (bytes = 0 for SV_F32 models), zero unless a bf16 GEMM found
 * the K slices of one output tile on different XCDs - the placement its cache-local reduction
 * relies on and checks on every call; non-zero means results are suspect.  Cleared by
 * sv_workspace_init. */
#define SV_WS_ATTN_OUT 0
#define SV_WS_Q 1
#define SV_WS_STATUS 2
int sv_workspace_region(const sv_model_cfg *cfg, int B, int T, int n_scored, int which,
                        size_t *offset, size_t *bytes);

/* Measurement aid: sv_verify_layer issued product by product (one launch each, the form that rows beyond 64
 * always take), which records the caller's HIP events on `stream`
 * around single kernel launches so that a benchmark can read per-kernel durations with
 * hipEventElapsedTime: events[0],[1] bracket the q/k/v GEMM, [2],[3] the tree attention,
 * [3],[4] the output GEMM, [5],[6] the gate/up GEMM, [7],[8] the down GEMM.
 * events: [host] array of SV_N_TIMING_EVENTS hipEvent_t (created by the caller with timing
 * enabled).  SV_ERR_NULL if the array or an entry is NULL. */
#define SV_N_TIMING_EVENTS 9
int sv_verify_layer_timed(const sv_model_cfg *cfg, const void *packed, float *x,
                          const sv_kv_view *kv, const sv_tree *tree, int B, void *workspace,
                          size_t ws_bytes, void *stream, void *const *events);

/* Measurement aid, no part of the verification path: reads `bytes` of device memory once with
 * the access pattern of the weight stream (16-byte non-temporal loads, 1 KiB per wave and
 * instruction, 8 KiB per wave in flight) and discards the data.  bench.py times it to report
 * the streaming-read rate the GPU reaches next to its data-sheet HBM peak.
 *   ptr: [device], 16-byte aligned, bytes a multiple of 16;  sink: [device] 16 bytes, 16-byte
 *   aligned (written only for one data pattern in 2^96)
 * SV_ERR_SHAPE for sizes or alignments outside that. */
int sv_stream_read(const void *ptr, size_t bytes, void *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SPECVLA_VERIFY_AUX_H */
