/*
 * deinfer_testing.h - test and measurement aids of the low-rank linear-layer library.
 *
 * Nothing here is part of the product surface (include/deinfer.h): these entry points exist so
 * that tests can force every kernel variant and a benchmark can time one internal launch or
 * measure what the device itself delivers.  The "set" calls change state of the CALLING THREAD
 * only (thread-local): calls of other threads are never affected.  None of them may be used
 * while the thread's stream is being captured into a graph with events set.
 */
#ifndef DEINFER_TESTING_H
#define DEINFER_TESTING_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * An entry-point call is several kernel launches (decode sizes: downward projection, reduce,
 * upward projection; prefill sizes: one GEMM per stage).  After this call the library records
 * start_event before, and stop_event after, every launch of the kind `which` that THIS THREAD
 * makes (both are hipEvent_t created with timing enabled, passed as void*), on the stream of the
 * call, so that a benchmark can time that one kernel with HIP events.  NULL events or
 * which == 0 switch it off (the default).
 */
enum {
  DEINFER_PROF_NONE = 0,
  DEINFER_PROF_DECODE_DOWN = 1,
  DEINFER_PROF_DECODE_REDUCE = 2,
  DEINFER_PROF_DECODE_UP = 3,
  DEINFER_PROF_PREFILL_DOWN = 4,
  DEINFER_PROF_PREFILL_UP = 5
};
int deinfer_set_profile_events(int which, void *start_event, void *stop_event);

/*
 * The workgroup tile of the compute-bound (T > 128) kernel for the calls of THIS THREAD.  0 (the
 * default) lets every launch choose: 256 tokens x 256 features; 128 x 256 while the larger tiles
 * of the launch would occupy at most half of the compute units; 128 x 128 while that still
 * holds for the 128 x 256 tiles; a launch of more than one round of 256 x 256 tiles whose last
 * round would be at most half full runs that round's feature blocks as 128 x 256 tiles in the
 * same launch.  deinfer_set_prefill_token_tile(128 or 256) forces the token extent for every
 * launch that has the choice (launches with a split k range always use 256),
 * deinfer_set_prefill_feature_tile(128 or 256) the feature extent of the 128-token tiles
 * (launches with the rotary epilogue always use 256); DEINFER_TOKEN_TILE_BOTH makes every such
 * launch run the second half of its feature blocks as 128 x 256 tiles.  Results do not depend on
 * the tile: each output element is the same sum taken in the same order.
 */
#define DEINFER_TOKEN_TILE_BOTH 384
int deinfer_set_prefill_token_tile(int tokens);
int deinfer_set_prefill_feature_tile(int features);

/*
 * The second stage of a GLU call of 17 to 128 tokens for the calls of THIS THREAD: 0 (the default)
 * lets every call choose between the launch that multiplies both products in one workgroup (no
 * partial sums; taken where its workgroups fill most of one round of the compute units) and the
 * split with partial sums and a combining launch; 1 forces the former, -1 the latter.
 */
int deinfer_set_decode_glu_one_launch(int mode);

/*
 * What this device delivers on the two rooflines of the path (Sec. 5.2 "Throughput Analysis"
 * reports throughput only; the denominators are this build's), for a benchmark that prints a
 * measured ceiling beside the published one.  Both enqueue one kernel on `stream`, allocate
 * nothing and do not synchronise.  sink: device scratch of at least DEINFER_PROBE_SINK_BYTES,
 * 16-byte aligned, contents undefined afterwards.
 *   deinfer_probe_stream_read  reads buf[0 .. bytes) once (bytes a positive multiple of 1024,
 *                              buf 16-byte aligned, device) with plain coalesced loads.
 *   deinfer_probe_mfma_bf16    every wavefront of a one-workgroup-per-compute-unit grid issues
 *                              8 * n_rounds bf16 32x32x16 matrix products back to back on register
 *                              operands taken from `operands` (device, >= 8192 bytes of bf16
 *                              values, 16-byte aligned); *flops_out (host, may be NULL) receives
 *                              the floating-point operations of the launch.
 */
#define DEINFER_PROBE_SINK_BYTES ((size_t)1 << 20)
int deinfer_probe_stream_read(const void *buf, size_t bytes, void *sink, size_t sink_bytes, void *stream);
int deinfer_probe_mfma_bf16(const void *operands, size_t operand_bytes, int64_t n_rounds,
                            void *sink, size_t sink_bytes, void *stream, double *flops_out);

#ifdef __cplusplus
}
#endif
#endif /* DEINFER_TESTING_H */
