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
 * 1 = the filtering scan wherever it exists, 2 = never.  The results are the same.  Process-wide;
 * not thread-safe against concurrent calls. */
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

#ifdef __cplusplus
}
#endif
#endif /* HG_ATTN_DEBUG_H */
