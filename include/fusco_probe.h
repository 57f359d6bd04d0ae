/*
 * fusco_probe.h - measurement aids of libfusco.so.  Not part of the shuffle's boundary (fusco.h):
 * plain copy and row-traffic kernels that show what the memory system gives for traffic of the
 * shuffle's shape, and per-call kernel timing without stream events.  Same conventions as fusco.h:
 * d_* are caller-owned device pointers, `stream` is a hipStream_t passed as void*, the return value
 * is FUSCO_OK or a negative FUSCO_ERR_*, nothing is allocated or synchronised.
 */
#ifndef FUSCO_PROBE_H
#define FUSCO_PROBE_H

#include "fusco.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Measurement aid: plain device copy of `bytes` bytes (multiple of 16) with the same 16-byte
 * accesses the shuffle kernels use.  Used to calibrate hardware traffic counters and as the
 * copy ceiling next to the shuffle's bandwidth.
 */
int fusco_probe_copy(void *d_dst, const void *d_src, size_t bytes, void *stream);

/*
 * Measurement aid: whole-row traffic of a chosen shape, with no plan behind it and no arithmetic.
 * One workgroup reads `reads_per_group` rows of d_src (XOR-ing them) and writes `writes_per_group`
 * rows of d_dst; supported shapes (reads, writes): (0,1) fill, (1,0) read, (1,1) copy, (1,8) the
 * dispatch mix, (8,1) the combine mix.  The grid is dst_rows / writes_per_group workgroups (for
 * (1,0): src_rows); dst_rows must be a multiple of writes_per_group and src_rows must hold
 * groups * reads_per_group rows.  scatter == 0 walks both buffers in launch order; otherwise row i of
 * a stream sits at (i * m) mod rows with m coprime to the row count, i.e. rows land far from their
 * launch-order neighbours as they do under routing.  write_through != 0 uses the write-through stores
 * of the combine kernel, else plain stores.  d_sink (one uint32 in device memory) is needed for
 * (1,0) only and is never written in practice.  Buffers: [src_rows, row_bytes], [dst_rows,
 * row_bytes], 16-byte aligned, row_bytes a multiple of 16.  Returns FUSCO_ERR_INVALID_ARG otherwise.
 */
int fusco_probe_rows(const void *d_src, uint32_t src_rows, void *d_dst, uint32_t dst_rows, size_t row_bytes,
                     int reads_per_group, int writes_per_group, int scatter, int write_through,
                     uint32_t *d_sink, void *stream);

/*
 * Measurement aid: kernel time without stream events between the kernels.  The next fusco_plan,
 * fusco_dispatch (fused modes), fusco_plan_dispatch or fusco_combine call made by the calling thread attaches the two HIP
 * events (hipEvent_t passed as void*, created with timing enabled) to its own kernels: start_event
 * is recorded when the call's first kernel begins, stop_event when its last kernel ends, both from
 * the kernels' own dispatch timestamps.  hipEventElapsedTime(start, stop) after the stream has been
 * synchronised is then the device time of that call, as a profiler's kernel trace reports it; a
 * pair of hipEventRecord calls around the launch would add the cost of the barriers they put into
 * the stream.  The arming is per thread and is used up by the first such call that launches
 * kernels (a call that fails its argument checks or has an empty layout leaves it armed;
 * FUSCO_DISPATCH_TWO_HOP uses it up without recording).  Events are not recorded into a stream
 * that is being captured: do not arm before a captured call.
 */
int fusco_probe_time_next_call(void *start_event, void *stop_event);

#ifdef __cplusplus
}
#endif
#endif /* FUSCO_PROBE_H */
