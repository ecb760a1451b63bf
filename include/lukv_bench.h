/*
 * lukv_bench.h - instrumentation and measurement helpers of liblukv, for programs that time the
 * path (bench.py).  Not part of the method; nothing in lukv.h depends on it.
 */
#ifndef LUKV_BENCH_H
#define LUKV_BENCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Stage timing (process-wide, not thread-safe).  While events are set, the main kernel of stage i
 * of every call is launched with events[2*i] as its start event and events[2*i+1] as its stop event (hipEvent_t,
 * created by the caller, passed as void*): hipEventElapsedTime(start, stop) is then that kernel's
 * own duration, as a profiler reports it.  Entries that are NULL or beyond n_events are skipped.
 * The array must stay valid until lukv_set_stage_events(NULL, 0).  Stages: allocate (the budget
 * kernel of a stand-alone lukv_allocate), score_stats, score_accum, pool (lukv_score only),
 * sel_head, sel_gather (selection in calls of at least 64 heads whose sequences have at most 32768
 * tokens), sel_hist, sel_tail, sel_emit (selection in every other call); lukv_stage_name gives the same names, "" when out of range. */
#define LUKV_NUM_STAGES 9
#define LUKV_NUM_STAGE_EVENTS (2 * LUKV_NUM_STAGES)
int lukv_set_stage_events(void* const* events, int32_t n_events);
const char* lukv_stage_name(int32_t stage);

/* Plain streaming kernels of known size: the achievable ceilings of this GPU, measured beside the
 * path's kernels and quoted next to the nominal HBM peak.
 *   lukv_bench_stream_read: every 16-byte word of src[0, bytes) is read once (grid-strided, eight
 *       loads in flight per thread) and folded into sink[4 * blocks] (4 bytes per wave).
 *   lukv_bench_copy: dst[0, bytes) = src[0, bytes), 16 bytes per lane.
 * src, dst device, 16-byte aligned; bytes a multiple of 16; blocks = workgroups of 256 threads to
 * launch, 1..65536; sink device, >= 16 * blocks bytes.  Enqueue only; LUKV_EINVAL otherwise. */
int lukv_bench_stream_read(const void* src, int64_t bytes, void* sink, int32_t blocks, void* stream);
int lukv_bench_copy(const void* src, void* dst, int64_t bytes, int32_t blocks, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LUKV_BENCH_H */
