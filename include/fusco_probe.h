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
 * Measurement aid: d_buf (bytes a multiple of 4096, 16-byte aligned) written (write != 0) or read as a stream
 * of 4 KiB pieces, one workgroup per piece, one 16-byte access per thread, with a chosen assignment of pieces
 * to the 8 XCDs of the GPU.  The hardware hands workgroups to the XCDs in turn, so workgroup b = 8 i + x runs on
 * XCD x; it takes piece ((i / run) * 8 + x) * run + i mod run, i.e. every XCD works through runs of run_pieces
 * consecutive pieces and the 8 runs of a round lie next to each other.  The bytes moved, and the address window
 * in flight across the chip, are the same for every run_pieces; only which XCD touches which piece changes.
 * run_pieces == 1 is plain launch order; pieces / 8 gives each XCD one contiguous eighth of the buffer.
 * Requires pieces % 8 == 0 and (pieces / 8) % run_pieces == 0.  scatter != 0 ignores run_pieces and sends
 * workgroup b to piece b * m mod pieces, m coprime to the piece count.  A written piece holds its own index in
 * word 0 of each 16-byte unit.  d_sink (one uint32 on the device) is needed for reads and never written in
 * practice.
 */
int fusco_probe_pieces(void *d_buf, size_t bytes, int write, uint32_t run_pieces, int scatter, uint32_t *d_sink,
                       void *stream);

/*
 * Validation aid: the consumer side of the slice protocol of fusco_segments_copy (the role a network engine
 * plays in the paper's pipelined workflow, section 3.2: it takes a slice as soon as the slice is ready).  One
 * workgroup, meant to run on another stream while fusco_segments_copy packs d_stream: it walks the
 * ceil(total_bytes / slice_bytes) slices in order, polls d_slice_fill[s] with acquire loads at system scope
 * until the count reaches the slice's size, and then adds up the slice's 32-bit words.  The kernel always
 * ends: it polls at most max_polls times in all (at most 2^24), after which the remaining slices are
 * reported as not ready.  d_report: [slices][4] uint32 = { seen complete (0/1), polls spent waiting for it, low
 * and high 32 bits of the 64-bit sum of the slice's 32-bit words }.  total_bytes must be the exact size of the
 * packed stream (a multiple of 16).  The caller zeroes d_slice_fill before launching the two sides.
 */
int fusco_probe_consume_slices(const void *d_stream, uint64_t total_bytes, uint64_t slice_bytes,
                               const uint32_t *d_slice_fill, uint32_t max_polls, uint32_t *d_report, void *stream);

/*
 * Study and test aid: which kernel every later fusco_dispatch of the process uses where it has a choice.
 * 0: automatic.  1: the token walk (one workgroup per token), also where the rows would be moved tile by tile in
 * transfer order.  2: the transfer order wherever its workgroup shape allows, also at sizes where the token walk
 * is preferred.  fusco_dispatch_in_transfer_order reflects the setting.  which < 0 only reads it.  Returns the
 * previous setting, FUSCO_ERR_INVALID_ARG for which > 2.  The result of fusco_dispatch does not depend on it.
 */
int fusco_probe_dispatch_kernel(int which);

/*
 * Study and test aid: loads and stores of fusco_dispatch's token walk.  0: automatic (plain stores and
 * non-temporal loads while the tensors it writes fit the 256 MB memory-side cache and FUSCO_DISPATCH_STREAMING
 * is not given; otherwise non-temporal stores, with cached loads for a source tensor of up to 128 MiB and
 * non-temporal loads for a larger one).  1: non-temporal loads, plain stores.  2: cached loads, plain stores.
 * 3: non-temporal loads and stores.  4: cached loads, non-temporal stores.  which < 0 only reads the setting.
 * Returns the previous setting, FUSCO_ERR_INVALID_ARG for which > 4.  The result of fusco_dispatch does not
 * depend on it.
 */
int fusco_probe_dispatch_walk(int which);

/*
 * Study and test aid: whether the tiled dispatch pulls a tile's source rows towards the L2 at the start of the
 * tile (its first workgroups each read one more row and drop it).  0: automatic (on when the source tensor is
 * taken in one piece).  1: off.  2: on.  which < 0 only reads the setting.  Returns the previous setting,
 * FUSCO_ERR_INVALID_ARG for which > 2.  The result of fusco_dispatch does not depend on it.
 */
int fusco_probe_dispatch_pull(int which);

/*
 * Study and test aid: how many workgroups of the tiled dispatch a compute unit holds at once.  0: automatic (5 to
 * 12, by the size of the rows or column segments, for rows of 4 KiB and more with a source tensor of at most
 * 116 MiB; no cap otherwise).  3 ... 15: that many (the launch asks for dynamic LDS it does not use, which caps the
 * number; 13 comes out as 14).  16: no cap.  wgs < 0 only reads the setting.  Returns the previous setting,
 * FUSCO_ERR_INVALID_ARG for 1, 2 and values above 16.  The result of fusco_dispatch does not depend on it.
 */
int fusco_probe_dispatch_occupancy(int wgs);

/*
 * Study and test aid: the largest source tensor (bytes of x plus its second plane) that fusco_dispatch's
 * tiled mode takes in one piece.  Larger ones are taken in chunks of whole rounds of 8 tiles whose source rows
 * fit this many bytes (at least 8 tiles), each chunk with launches of its own: a sequential read of the chunk's
 * source rows, which leaves them in the 256 MB memory-side cache, then the chunk's tiles.  bytes = 0 only
 * reads the value; otherwise the value is replaced, for the whole process, and the previous one returned.
 * The default is 128 MiB.  The result of fusco_dispatch does not depend on it.
 */
size_t fusco_probe_source_chunk_bytes(size_t bytes);

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
