/*
 * fusco.h - C boundary of the MI355X (gfx950) MoE token shuffle with the layout transformation
 * fused into the data movement.
 *
 * The library turns the router's token-expert matrix into a two-level layout descriptor
 * (fusco_plan), moves token rows straight to their final expert-major rows (fusco_dispatch) and
 * brings expert outputs back into token order with the gate weights (fusco_combine).
 *
 * Conventions for every entry point
 *   - Pointers named d_* are DEVICE pointers into memory owned by the caller.  The library never
 *     allocates, frees or keeps device memory, and never synchronises: each call only enqueues
 *     kernels on `stream` (a hipStream_t passed as void*; NULL is the default stream).
 *   - Device pointers must be 16-byte aligned.  Buffers must not overlap, except that the y
 *     argument of fusco_combine may be the expert buffer fusco_dispatch wrote.
 *   - Return value: FUSCO_OK (0) when the work was enqueued, a negative FUSCO_ERR_* otherwise.
 *     On an error nothing is launched.
 *   - A layout with N == 0 is valid everywhere: sizes are still checked, tensor pointers (all of
 *     them empty then) may be NULL, nothing is launched by the movers and FUSCO_OK is returned.
 *   - Expert-parallel devices are D virtual partitions of one GPU's buffers.  Expert e lives on
 *     device e / (E / D) (contiguous placement; E must be a multiple of D).
 *   - All row orders are deterministic: rows of one expert, and rows of one device's receive
 *     tensor, are in ascending token order.
 */
#ifndef FUSCO_H
#define FUSCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FUSCO_VERSION 110

#define FUSCO_OK 0
#define FUSCO_ERR_INVALID_ARG (-1) /* null pointer, size out of range, misaligned pointer or row size */
#define FUSCO_ERR_WORKSPACE (-2)   /* caller-provided memory too small                               */
#define FUSCO_ERR_UNSUPPORTED (-3) /* dtype or flag combination not implemented                       */
#define FUSCO_ERR_HIP (-4)         /* the HIP runtime refused a launch                                */
#define FUSCO_ERR_STATIC_LIMIT (-5) /* fusco_plan_static: the input needs more scratch than the static buffer */

#define FUSCO_MAX_K 64   /* experts per token                    */
#define FUSCO_MAX_E 1024 /* experts (and therefore devices)      */
#define FUSCO_MAX_ROW_BYTES (1u << 20) /* one row of the movers, both planes of a dispatch together */
#define FUSCO_STATIC_SCRATCH_BYTES (4u << 20) /* planner scratch held by the library for fusco_plan_static */

/* element types of fusco_combine */
#define FUSCO_BF16 0
#define FUSCO_F32 1

/* flags of fusco_dispatch (no tensor flag means FUSCO_DISPATCH_EXPERT) */
#define FUSCO_DISPATCH_EXPERT 1u /* write the expert-activation tensor (level 2 result)       */
#define FUSCO_DISPATCH_WIRE 2u   /* write the deduplicated per-device receive tensors (level 1) */
#define FUSCO_DISPATCH_TWO_HOP 4u /* hop by hop: x -> receive tensors -> expert tensor (implies both) */
#define FUSCO_DISPATCH_STREAMING 8u /* modifier: write the rows past the memory-side cache (see fusco_dispatch) */

/*
 * Layout descriptor: the two-level descriptor lists of the paper's Communication Planner
 * (section 3.3, the paragraph on the descriptor-level plan) for fixed-size segments.  A segment is one
 * token row, so a segment descriptor (address, size) collapses to a row index.
 *
 * N tokens, k experts per token, E experts, D devices, P = N * k (token, expert) pairs.
 * Pair index p = t * k + j.  "slot" = row in the expert-activation tensor [P rows], ordered by
 * device, then expert, then token.  "send row" = row in the concatenated per-device receive
 * tensors [U rows, U = send_off[D]], ordered by device, then token; a token has one send row per
 * distinct destination device (first appearance of the device among its k entries).
 * All arrays live in device memory carved by fusco_layout_bind.
 */
typedef struct fusco_layout {
    int32_t N, k, E, D, P;
    int32_t send_cap;        /* rows reserved for send_src and a wire buffer: N * min(k, D)          */
    int32_t *exp_count;      /* [E]    rows per expert                                                */
    int32_t *exp_off;        /* [E+1]  exclusive prefix sum of exp_count; exp_off[E] == P             */
    int32_t *send_count;     /* [D]    send rows per device                                           */
    int32_t *send_off;       /* [D+1]  exclusive prefix sum of send_count; send_off[D] == U           */
    int32_t *pair_slot;      /* [P]    pair -> slot                 (level-2 receive descriptor)      */
    int32_t *slot_pair;      /* [P]    slot -> pair                                                   */
    int32_t *slot_token;     /* [P]    slot -> token                (source-token index)              */
    int32_t *send_src;       /* [send_cap] send row -> token; rows >= U are not written (level-1 send) */
    int32_t *pair_send_row;  /* [P]    pair -> send row of (t, device of its expert) (level-2 send)   */
    int32_t *slot_send_row;  /* [P]    slot -> send row holding its payload                           */
    uint8_t *pair_first;     /* [P]    1 iff the pair is the first appearance of its device in token t */
    int32_t *status;         /* [1]    number of expert ids outside [0, E) seen by the last fusco_plan */
    /* Transfer order (section 3.2: descriptor lists are dense arrays in transfer order).  The tokens are cut
     * into tile_count tiles of tile_tokens consecutive tokens (the last one may hold fewer); the entries
     * [i * tile_tokens * k, (i + 1) * tile_tokens * k) list the slots of tile i's (token, expert) pairs in
     * ascending order, i.e. expert by expert with ascending tokens inside an expert, followed by -1 up to the
     * tile's capacity (a ragged last tile, pairs with an invalid expert id).  fusco_dispatch moves the rows
     * in this order, tile by tile.  tile_tokens and tile_count depend on N and k only and are set by
     * fusco_layout_bind. */
    int32_t *tile_slots;     /* [tile_count * tile_tokens * k]                                        */
    int32_t tile_tokens, tile_count;
} fusco_layout;

/* Library version (FUSCO_VERSION of the build). */
int fusco_version(void);

/* Static text for a FUSCO_* return code. */
const char *fusco_status_string(int status);

/*
 * Bytes of device memory the descriptor arrays need for these sizes (0 if the sizes are
 * invalid: N < 0, k outside [1, FUSCO_MAX_K], E outside [1, FUSCO_MAX_E], D < 1, E % D != 0,
 * or N * k >= 2^31).
 */
size_t fusco_layout_bytes(int32_t N, int32_t k, int32_t E, int32_t D);

/* Bytes of planner scratch (partial counts per tile of 1024 or 2048 pairs and per chunk of tiles) for
 * these sizes; 0 if the sizes are invalid. */
size_t fusco_scratch_bytes(int32_t N, int32_t k, int32_t E, int32_t D);

/*
 * Fill *L (host struct) with the sizes and with pointers carved out of the caller's device
 * block d_mem of `bytes` bytes (256-byte aligned base).  Host-only: touches no device memory.
 * Errors: FUSCO_ERR_INVALID_ARG (null, bad sizes, misaligned), FUSCO_ERR_WORKSPACE (too small).
 */
int fusco_layout_bind(fusco_layout *L, int32_t N, int32_t k, int32_t E, int32_t D, void *d_mem, size_t bytes);

/*
 * Planner (section 3.3): per-expert histogram, prefix-scan offsets, stable expert-major slot of
 * every (t, e) pair, and removal of duplicate (token, device) sends with the resulting send rows.
 * d_topk_idx: [N, k] int32 row-major, the token-expert matrix A (may be NULL when N == 0).
 * Ids outside [0, E) are counted in L->status, get pair_slot = pair_send_row = -1 and are skipped
 * by dispatch and combine; the plan is then not a valid layout (slots at the end of the tensor
 * stay unassigned).
 * d_scratch: at least fusco_scratch_bytes() bytes, contents irrelevant before and after.
 * Every descriptor array is fully rewritten (send_src only in rows < U).  N == 0 is allowed.
 */
int fusco_plan(fusco_layout *L, const int32_t *d_topk_idx, void *d_scratch, size_t scratch_bytes, void *stream);

/*
 * fusco_plan for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  Same arguments and results as fusco_plan,
 * but the planner's scratch (per-tile and per-chunk counts) is a static array of FUSCO_STATIC_SCRATCH_BYTES
 * (4 MiB) inside the library, present on every GPU the library runs on until the process ends.  The call
 * allocates and frees nothing.  Inputs whose fusco_scratch_bytes() exceeds that size are refused with
 * FUSCO_ERR_STATIC_LIMIT and nothing is launched (4 MiB covers about 7.9 million (token, expert) pairs at
 * E + D = 264, e.g. 990 000 tokens with k = 8); use fusco_plan with a workspace of your own for those.
 * The first call on a device looks up the address of that device's copy of the array (no allocation; make
 * that first call outside a graph capture); the device current at the call must be the one `stream` belongs to.
 * All calls on one GPU share the one array: two fusco_plan_static calls that may overlap on the same GPU
 * (different streams, no ordering between them) race on it and give undefined descriptors; calls in one
 * stream, or ordered by events, are safe.  The array needs no clearing: every call writes all counts it reads.
 * Errors otherwise as fusco_plan; FUSCO_ERR_HIP also when the array's address cannot be resolved.
 */
int fusco_plan_static(fusco_layout *L, const int32_t *d_topk_idx, void *stream);

/*
 * Fused gather-pack (section 3.2, intra-node path: descriptor interpretation inlined into the
 * copy, no intermediate pass): every token row is read once and written to each of its slots,
 *     expert_buf[pair_slot[t*k+j]] = x[t]                          (FUSCO_DISPATCH_EXPERT)
 *     send_buf[pair_send_row[t*k+j]] = x[t] where pair_first       (FUSCO_DISPATCH_WIRE)
 * For large inputs the expert tensor is written tile by tile in the layout's transfer order (see
 * fusco_dispatch_in_transfer_order): every XCD of the GPU takes whole tiles of tokens and writes their rows
 * expert by expert with streaming stores, the tile's source rows being read from memory once and from the
 * XCD's L2 afterwards while they stay there.  A source tensor of more than 128 MiB is taken in chunks of tiles,
 * each chunk after a sequential read of its source rows (a few launches instead of one).  Otherwise every
 * token's row is read once and stored to its k rows at once (token walk).
 * Rows are opaque bytes.  d_x: [N, row_bytes], row_bytes a positive multiple of 16.  An optional
 * second plane (e.g. per-block scales of an fp8 payload) of aux_row_bytes (multiple of 16, or 0
 * with NULL aux pointers) follows the same descriptors; row_bytes + aux_row_bytes may not exceed
 * FUSCO_MAX_ROW_BYTES.  d_expert_buf: [P, row_bytes],
 * d_expert_aux: [P, aux_row_bytes]; d_send_buf: [send_cap, row_bytes], d_send_aux likewise; rows
 * >= U of the send buffers are not written.  Buffers of a plane that is not requested by `flags`
 * may be NULL.
 * FUSCO_DISPATCH_TWO_HOP executes the two descriptor levels one after the other, as the planner
 * describes them (section 3.3): first one row per (token, device) into the receive tensors, then
 *     expert_buf[s] = send_buf[slot_send_row[s]]
 * for every assigned slot.  Both tensors are written and hold the same bytes as in the fused mode;
 * the extra pass costs U + P more row reads.
 * FUSCO_DISPATCH_STREAMING may be added to the fused modes (not to FUSCO_DISPATCH_TWO_HOP): the token walk then
 * writes its rows with non-temporal stores, which do not stay in the GPU's 256 MB memory-side cache (the
 * transfer order always writes that way, and so does the token walk on its own when the tensors it writes
 * exceed that cache).  Choose it for smaller tensors when other traffic (an expert computation) comes between
 * this call and the first reader of the rows: a plain dispatch leaves its rows dirty in that cache, and whoever
 * streams through memory next pays for writing them back.  Results are identical either way.
 */
int fusco_dispatch(const fusco_layout *L, const void *d_x, size_t row_bytes, const void *d_x_aux,
                   size_t aux_row_bytes, void *d_expert_buf, void *d_expert_aux, void *d_send_buf,
                   void *d_send_aux, uint32_t flags, void *stream);

/*
 * Host-only: 1 if fusco_dispatch with these row sizes and flags moves the rows tile by tile in the layout's
 * transfer order (tile_slots), 0 if it walks the tokens, negative on invalid arguments.  The transfer order
 * is used when only the expert tensor is written, k >= 2, the layout has at least 16 tiles, and the source
 * rows of one tile (tile_tokens * (row_bytes + aux_row_bytes)) fit the 4 MB L2 of an XCD whole (at most
 * 3840 KiB) or cut into up to eight column segments of at least 4 KiB each, which are then moved in as many
 * passes over the tile; and when the sizes make it pay: the expert tensor is larger than the 256 MB memory-side cache
 * (a smaller one is left there by the token walk's plain stores for its reader), rows shorter than 8 KiB
 * come with a source tensor of at most 128 MiB (less than 128 MiB for rows shorter than 4 KiB), and a source
 * tensor of more than 128 MiB comes with k >= 8, or with k >= 5 and rows that need no column segments.  Both
 * ways write the same bytes.
 */
int fusco_dispatch_in_transfer_order(const fusco_layout *L, size_t row_bytes, size_t aux_row_bytes, uint32_t flags);

/*
 * fusco_plan followed by fusco_dispatch (FUSCO_DISPATCH_EXPERT only) in a single launch, for inputs
 * that fit one planner tile: N <= floor(2048 / k) tokens (decode-sized batches, where a chain of
 * dependent launches costs more than the work; the planner's cost is fixed and shows at small
 * sizes, section 5.2).  Results are exactly those of the two calls: every descriptor array of *L is
 * written as by fusco_plan (no scratch is needed), d_expert_buf / d_expert_aux as by fusco_dispatch.
 * Arguments as in those two calls.  Returns FUSCO_ERR_UNSUPPORTED when the input needs more than
 * one tile; the caller then makes the two calls.
 */
int fusco_plan_dispatch(fusco_layout *L, const int32_t *d_topk_idx, const void *d_x, size_t row_bytes,
                        const void *d_x_aux, size_t aux_row_bytes, void *d_expert_buf, void *d_expert_aux,
                        void *stream);

/*
 * Weighted combine (reverse path of the shuffle: weighted sum of a token's expert outputs,
 * section 2.1):   out[t, :] = sum_{j=0..k-1} w[t, j] * y[pair_slot[t*k+j], :]
 * accumulated in fp32 with one fused multiply-add per term in ascending j from +0, then rounded
 * once (nearest even) when out_dtype is FUSCO_BF16.
 * d_y: [P, H] of y_dtype, d_w: [N, k] fp32, d_out: [N, H] of out_dtype.  H * sizeof(y element)
 * must be a multiple of 16 and at most FUSCO_MAX_ROW_BYTES.  `flags` must be 0.
 */
int fusco_combine(const fusco_layout *L, const void *d_y, int y_dtype, const float *d_w, void *d_out,
                  int out_dtype, int32_t H, uint32_t flags, void *stream);

/*
 * Combine along the two descriptor levels in reverse (mirror of FUSCO_DISPATCH_TWO_HOP; the paper
 * only says the reverse path is symmetric, the arithmetic is this library's reading):
 *   partial[r, :] = sum over the entries j of token send_src[r] whose send row is r of
 *                   w[t, j] * y[pair_slot[t*k+j], :]      fp32 fused multiply-adds, ascending j, from +0
 *   out[t, :]     = sum of the token's partial rows        fp32 additions from +0, in the order in which
 *                                                          the devices first appear among the k entries
 * so one fp32 row per (token, device) would cross the link instead of one row per (token, expert).
 * d_partial: [send_cap, H] fp32 scratch tensor, rows < U are overwritten.  H must be a multiple of 4
 * (and H * sizeof(y element) a multiple of 16).  The result differs from fusco_combine only by the
 * association of the sum: at most (k + D) * 2^-24 * sum_j |w_j y_j| from the exact value.
 */
int fusco_combine_two_hop(const fusco_layout *L, const void *d_y, int y_dtype, const float *d_w, float *d_partial,
                          void *d_out, int out_dtype, int32_t H, void *stream);

/*
 * Disaggregated baseline: the multi-stage shuffle the paper starts from (section 1: rearrange by
 * destination rank, all-to-all, rearrange by expert, and the symmetric reverse; section 5.4, the
 * "dComm-off" ablation, performs the rearrangements explicitly around the transfer).  Each stage is
 * a separate pass over the whole buffer; no deduplication (one row per (token, expert) pair).  It
 * exists to measure what fusing buys on this GPU and produces the same expert tensor / output.
 *
 * fusco_disaggregated_plan fills Lr, a second layout bound by the caller with
 * fusco_layout_bind(Lr, N, k, D, D, ...): the stable order of the pairs by destination device
 * ("rank-major": Lr->pair_slot is the pair's row, Lr->slot_token its token).  d_topk_dev: [N, k]
 * int32 scratch that receives the device of every pair.  d_scratch as for fusco_plan with (N,k,D,D).
 * L must already hold the plan of the same d_topk_idx.
 *
 * fusco_disaggregated_dispatch: stage_a[r] = x[token of rank row r]; stage_b = stage_a (the
 * exchange between virtual devices, a contiguous copy); expert_buf[s] = stage_b[rank row of slot s].
 * fusco_disaggregated_combine: stage_b[r] = y[slot of rank row r]; stage_a = stage_b;
 * out[t] = sum_j w[t,j] * stage_a[rank row of (t,j)] (same arithmetic as fusco_combine).
 * d_stage_a, d_stage_b: [P, row] scratch tensors, overwritten.
 */
int fusco_disaggregated_plan(fusco_layout *Lr, const fusco_layout *L, const int32_t *d_topk_idx, int32_t *d_topk_dev,
                             void *d_scratch, size_t scratch_bytes, void *stream);
int fusco_disaggregated_dispatch(const fusco_layout *L, const fusco_layout *Lr, const void *d_x, size_t row_bytes,
                                 void *d_stage_a, void *d_stage_b, void *d_expert_buf, void *stream);
int fusco_disaggregated_combine(const fusco_layout *L, const fusco_layout *Lr, const void *d_y, int y_dtype,
                                const float *d_w, void *d_stage_a, void *d_stage_b, void *d_out, int out_dtype,
                                int32_t H, void *stream);

/*
 * Input of the load balancer (section 3.4): the cross-node traffic load of the GPU that owns this plan,
 * i.e. the volume it must transmit to remote nodes.  The D destination devices are grouped into nodes of
 * devices_per_node consecutive devices (D must be a multiple); the GPU itself sits on node home_node.
 *     *d_load = row_bytes * sum of send_count[d] over the devices d with d / devices_per_node != home_node
 * in bytes, after duplicate removal (one send row per token and destination device; plan with D = number
 * of nodes for the paper's one copy per node).  d_load: one int64 in device memory, 8-byte aligned, e.g. the
 * GPU's cell of the [nodes, gpus] matrix that fusco_balance_groups takes once every GPU has filled its own.
 * Must follow the fusco_plan of the same layout in stream order.  One small launch.
 */
int fusco_cross_node_load(const fusco_layout *L, int32_t devices_per_node, int32_t home_node, size_t row_bytes,
                          int64_t *d_load, void *stream);

/*
 * Online Group-Balanced Assignment (Algorithm 1, section 3.4).  Host-only, no GPU work.
 * load: [nodes, gpus] row-major, cross-node traffic load of every GPU.  For every node the GPUs are
 * sorted by descending load (equal loads keep ascending GPU index), the sorted list is rotated by
 * the node index, and communication group i takes the GPU at position i of every node's rotated
 * list: group_gpu[i * nodes + n] = sorted_n[(i + n) mod gpus], for gpus groups of one GPU per node.
 * The direction of the rotation and the tie order are not fixed by the paper; these are this
 * library's readings.  O(gpus^2) per node (gpus is 4..8 in practice).
 * Errors: FUSCO_ERR_INVALID_ARG (null, sizes < 1 or nodes * gpus > 2^24), FUSCO_ERR_WORKSPACE (host allocation failed).
 */
int fusco_balance_groups(const int64_t *load, int32_t nodes, int32_t gpus, int32_t *group_gpu);

/*
 * Segment descriptor (section 3.2): where a logical segment lies, as a byte offset from a base
 * pointer, and its size in bytes.  Offsets and sizes must be multiples of 16.  A descriptor list is
 * a dense array in transfer order; the sender's and the receiver's lists map one to one.
 */
typedef struct fusco_segment {
    uint64_t offset;
    uint64_t size;
} fusco_segment;

/*
 * Cumulative bytes of a descriptor list: d_cum[0] = 0, d_cum[i+1] = d_cum[i] + size of segment i
 * (d_cum has n + 1 entries).  The engine finds the segment of a stream position from this array.
 * Descriptors with an offset or size that is not a multiple of 16 are counted in *d_status and take
 * part with size 0.  n <= 2^26.  One launch, one workgroup.
 */
int fusco_segments_scan(const fusco_segment *d_desc, int64_t n, uint64_t *d_cum, int32_t *d_status, void *stream);

/*
 * Descriptor-driven transfer of n segments (section 3.2): segment i is read at d_src + the
 * sender's offset and written at d_dst + the receiver's offset; its size comes from d_cum (built
 * by fusco_segments_scan from either list: the lists must agree on sizes).  A NULL descriptor list
 * means that side is the contiguous stream, i.e. segment i starts at d_cum[i]: with d_dst_desc ==
 * NULL the segments are gathered and packed into one buffer (sender side, slices for the network),
 * with d_src_desc == NULL a packed buffer is scattered to its final places (receiver side).
 * src_bytes / dst_bytes: sizes of the two buffers; a 16-byte unit that would fall outside, or is
 * misaligned, is skipped and counted in *d_status (which this call only adds to: it continues the
 * count of fusco_segments_scan).  stream_capacity: upper bound of the total size known on the
 * host (the exact total is read on the device from d_cum[n]).
 * Slices: if d_slice_fill is given, the contiguous stream is cut into slices of slice_bytes (a
 * multiple of 16384) and d_slice_fill[s] counts the bytes of slice s that have been written and are
 * visible: the data is stored write-through at system scope, every workgroup waits for its stores
 * and only then adds its bytes with a system-scope atomic.  A consumer (another stream, another
 * agent) takes slice s once the count reaches min(slice_bytes, total - s * slice_bytes); it must
 * read the counter with an acquire (or bypass its caches for the slice's bytes).  Units skipped for
 * being out of range are not counted, so a slice with holes never becomes ready.  The counters are
 * reset to 0 by a small kernel at the start of the call, in stream order: a consumer that is still
 * polling the counters of the previous call on the same d_slice_fill races with that reset; give
 * overlapping transfers counter arrays of their own.
 */
int fusco_segments_copy(const void *d_src, uint64_t src_bytes, const fusco_segment *d_src_desc, void *d_dst,
                        uint64_t dst_bytes, const fusco_segment *d_dst_desc, const uint64_t *d_cum, int64_t n,
                        uint64_t stream_capacity, uint64_t slice_bytes, uint32_t *d_slice_fill, int32_t *d_status,
                        void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FUSCO_H */
