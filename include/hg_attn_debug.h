/*
 * hg_attn_debug.h -- tuning knobs and measurement aids of the partitioned decode-attention library.
 *
 * Nothing here is part of the method (include/hg_attn.h is): these calls exist so that tests can
 * reach every code path at small sizes (forced span lengths, forced top-k mode) and so that a
 * benchmark can time one kernel by itself.  The knobs are process-wide mutable state and are not
 * thread-safe against concurrent calls into the library; production callers leave them alone.
 * Unlike the calls of hg_attn.h, hg_attn_profile_times and hg_attn_profile_stop wait for the device.
 */
#ifndef HG_ATTN_DEBUG_H
#define HG_ATTN_DEBUG_H

#include "hg_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Tuning knob: force the span length in tokens (multiple of 64, 64..2^24); 0 restores the
 * built-in choice (one workgroup per compute unit on long inputs).  Process-wide; not
 * thread-safe against concurrent calls. */
hg_status hg_attn_set_span_tokens(int32_t span_tokens);

/* Tuning knob for hg_attn_topk: 0 = the library chooses between the filtering scan and the
 * two-call sequence (with one query head per KV head the scan needs long groups, on average at
 * least 128 tokens per kept token; with grouped queries it needs four or more query heads per
 * KV head and ranges long enough for several workgroups -- two for top_k <= 96, three for <= 144,
 * six for 256 -- to share each (range, KV head) pair),
 * 1 = the filtering scan wherever it exists, 2 = never, 3 = as 1, but with the survivors gathered
 * into dense lists and selected by the staged kernels (what the library does by itself only when
 * the lists of a group do not fit the one-launch selection: very many ranges per group, groups
 * beyond 2^20 tokens).  The results are the same.  Process-wide; not thread-safe against
 * concurrent calls. */
hg_status hg_attn_set_topk_mode(int32_t mode);

/*
 * Measurement aid: time the streaming kernel (the one that reads K and V) by itself.  After
 * hg_attn_profile_start(n, repeat), each of the next n hg_attn_partial / hg_attn_full calls
 * records a pair of HIP events on the caller's stream directly around that kernel, which is
 * launched `repeat` times back to back between the two events (it is idempotent), so that the
 * fixed cost of recording events is spread over several launches; results are unchanged.
 * hg_attn_profile_times waits for the events recorded so far and writes, for each of the first
 * min(calls, capacity) timed calls, the milliseconds of ONE launch (elapsed time / repeat) to
 * ms_each (HOST); *calls receives the number of timed calls.  hg_attn_profile_stop waits for the
 * events, returns the summed elapsed milliseconds and the number of kernel launches timed, and
 * switches the mode off.  Both block; process-wide; not thread-safe.
 */
hg_status hg_attn_profile_start(int32_t max_calls, int32_t repeat);
hg_status hg_attn_profile_times(float *ms_each, int32_t capacity, int32_t *calls);
hg_status hg_attn_profile_stop(float *total_ms, int32_t *launches);

/*
 * Measurement aid: a plain device copy of `bytes` bytes (multiple of 16; dst, src DEVICE,
 * 16-byte aligned, not overlapping).  Its HBM traffic is known exactly (bytes read, bytes
 * written), which makes it the reference that profiler byte counters are scaled by.
 */
hg_status hg_attn_calibration_copy(void *dst, const void *src, size_t bytes, void *stream);

/*
 * Measurement aid: a one-pass read stream with the access pattern of the streaming kernels (one
 * workgroup of 256 threads per compute unit, non-temporal 16-byte loads, 32 KiB per workgroup
 * iteration, the workgroups' shares starting 32 KiB further apart than they are long), alone or
 * next to writes.  It shows what this memory system gives such a stream -- the practical ceiling
 * the kernels are tuned against -- and what writes next to it cost.
 *
 *   src, read_bytes   DEVICE, 16-byte aligned; the kernel reads floor(read_bytes / 16 / CUs / 2048)
 *                     * 2048 vectors per workgroup; src must hold read_bytes + CUs * 32 KiB.
 *                     Fill it with zeros.
 *   dst               DEVICE, 16-byte aligned, or NULL when nothing is written; must hold
 *                     iterations * write_vectors_per_iteration * 16 bytes per workgroup
 *                     (at most read_bytes * write_vectors_per_iteration / 2048 in all) and 16 bytes at least.
 *   write_vectors_per_iteration   0 .. 2048: 16-byte vectors written per 32 KiB read, on average
 *                     (32 = 1/64 of the bytes, 256 = 1/8).
 *   burst_iterations  >= 1: the writes of that many iterations go out together, as one contiguous
 *                     run per workgroup (1 = a trickle; a burst that never completes is not written).
 *   streaming_stores  non-zero: non-temporal stores.
 */
hg_status hg_attn_calibration_stream(const void *src, size_t read_bytes, void *dst, int32_t write_vectors_per_iteration,
                                     int32_t burst_iterations, int32_t streaming_stores, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HG_ATTN_DEBUG_H */
