/*
 * CPU oracle for the MoE token shuffle with fused layout transformation.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the HIP library is
 * checked against.  It shares no code, header, table or helper with the HIP path and nothing
 * in the product may call it: only the tests, the smoke check and the benchmark's CPU-baseline
 * leg do.
 *
 * What it follows (paper section 3.3, the paragraph on the descriptor-level plan, and section 3.2,
 * the transfer engine):
 *   - A is the token-expert matrix (T x K): the experts the router assigned to each token.
 *   - B is the token-node matrix derived from A under a fixed expert placement.  Here a "node"
 *     is one virtual expert-parallel device, experts are placed in contiguous blocks, so the
 *     destination of expert e is e / (E / D).
 *   - Level 1, node-level forwarding descriptors: walk the tokens in order; for every
 *     destination n in B[t], the token gets one send descriptor in n's list at the first
 *     appearance of n in B[t] only.  The receiver's descriptor is the row of the token in
 *     n's receive tensor.
 *   - Level 2, expert-level distribution descriptors: for every (t, e) pair, the send
 *     descriptor is the token's row in the receive tensor of e's device after level 1, and the
 *     receive descriptor is the pair's exact row in the expert-activation tensor.
 *   - The transfer engine moves each segment (one token row) from the address in the send
 *     descriptor to the address in the receive descriptor.
 *   - The reverse path restores token order; the expert outputs of a token are combined by a
 *     weighted sum (section 2.1).
 *
 * Readings where the paper is silent:
 *   - rows inside one expert's segment, and inside one device's receive tensor, are in
 *     ascending token order (the planner walks the tokens and appends);
 *   - the receive tensors of the D devices are laid out one after the other (device-major), and
 *     so are the expert segments (device-major, then expert-major: with contiguous placement
 *     this is plain ascending expert id);
 *   - the weighted sum runs over the k entries of a token in their input order j = 0..k-1.
 *
 * Parity pins (tests/test_oracle_*.py): brute force from the definitions on tiny inputs, stable
 * argsort, a hand-worked example, structural invariants, special cases D = 1 and D = E, the
 * closed-form expected number of send rows, dyadic-weight and one-hot closed forms for the
 * weighted sum, and an fp64 library cross-check.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_MEM (-2)

#define ORACLE_BF16 0
#define ORACLE_F32 1

/* a growable list of int32 */
typedef struct {
    int32_t *v;
    int32_t n, cap;
} ilist;

static int ilist_push(ilist *l, int32_t x)
{
    if (l->n == l->cap) {
        int32_t cap = l->cap ? 2 * l->cap : 16;
        int32_t *v = (int32_t *)realloc(l->v, (size_t)cap * sizeof(int32_t));
        if (!v) return ORACLE_ERR_MEM;
        l->v = v;
        l->cap = cap;
    }
    l->v[l->n++] = x;
    return ORACLE_OK;
}

static void ilists_free(ilist *l, int32_t n)
{
    if (!l) return;
    for (int32_t i = 0; i < n; ++i) free(l[i].v);
    free(l);
}

/*
 * Planner.  Inputs: A[T*K] (row-major), T tokens, K experts per token, E experts, D devices.
 * Outputs (all caller-allocated):
 *   exp_count[E], exp_off[E+1]    rows per expert and their exclusive prefix sum
 *   send_count[D], send_off[D+1]  rows per device receive tensor and their prefix sum
 *   pair_slot[T*K]                (t,j) -> row in the expert-activation tensor
 *   slot_pair[T*K], slot_token[T*K]   inverse map and the token of each row
 *   send_src[T*min(K,D)]          receive-tensor row -> token (rows >= send_off[D] untouched)
 *   pair_send_row[T*K]            (t,j) -> row of token t in the receive tensor of dev(A[t,j])
 *   slot_send_row[T*K]            same, indexed by expert-activation row
 *   pair_first[T*K]               1 iff (t,j) is the first appearance of its device in B[t]
 */
int fusco_oracle_plan(const int32_t *A, int32_t T, int32_t K, int32_t E, int32_t D,
                      int32_t *exp_count, int32_t *exp_off,
                      int32_t *send_count, int32_t *send_off,
                      int32_t *pair_slot, int32_t *slot_pair, int32_t *slot_token,
                      int32_t *send_src, int32_t *pair_send_row, int32_t *slot_send_row,
                      uint8_t *pair_first)
{
    if (!A || T < 0 || K <= 0 || E <= 0 || D <= 0 || E % D != 0) return ORACLE_ERR_ARG;
    const int32_t Eloc = E / D;
    for (int64_t p = 0; p < (int64_t)T * K; ++p)
        if (A[p] < 0 || A[p] >= E) return ORACLE_ERR_ARG;

    int rc = ORACLE_OK;
    ilist *node_list = (ilist *)calloc((size_t)D, sizeof(ilist));   /* level 1: tokens per device */
    ilist *expert_list = (ilist *)calloc((size_t)E, sizeof(ilist)); /* level 2: pairs per expert  */
    int32_t *pos_in_node = (int32_t *)malloc((size_t)(T > 0 ? T : 1) * (size_t)K * sizeof(int32_t));
    if (!node_list || !expert_list || !pos_in_node) { rc = ORACLE_ERR_MEM; goto done; }

    /* Level 1: node-level forwarding descriptors, deduplicated at first appearance. */
    for (int32_t t = 0; t < T && rc == ORACLE_OK; ++t) {
        for (int32_t j = 0; j < K; ++j) {
            const int32_t n = A[(int64_t)t * K + j] / Eloc;          /* B[t][j] */
            int first = 1;
            int32_t j_first = j;
            for (int32_t i = 0; i < j; ++i)
                if (A[(int64_t)t * K + i] / Eloc == n) { first = 0; j_first = i; break; }
            pair_first[(int64_t)t * K + j] = (uint8_t)first;
            if (first) {
                pos_in_node[(int64_t)t * K + j] = node_list[n].n;
                rc = ilist_push(&node_list[n], t);
                if (rc != ORACLE_OK) break;
            } else {
                pos_in_node[(int64_t)t * K + j] = pos_in_node[(int64_t)t * K + j_first];
            }
        }
    }
    if (rc != ORACLE_OK) goto done;

    /* receive tensors of the devices, one after the other */
    send_off[0] = 0;
    for (int32_t n = 0; n < D; ++n) {
        send_count[n] = node_list[n].n;
        send_off[n + 1] = send_off[n] + node_list[n].n;
        for (int32_t i = 0; i < node_list[n].n; ++i) send_src[send_off[n] + i] = node_list[n].v[i];
    }

    /* Level 2: expert-level distribution descriptors. */
    for (int32_t t = 0; t < T && rc == ORACLE_OK; ++t)
        for (int32_t j = 0; j < K; ++j) {
            rc = ilist_push(&expert_list[A[(int64_t)t * K + j]], t * K + j);
            if (rc != ORACLE_OK) break;
        }
    if (rc != ORACLE_OK) goto done;

    exp_off[0] = 0;
    for (int32_t e = 0; e < E; ++e) {
        exp_count[e] = expert_list[e].n;
        exp_off[e + 1] = exp_off[e] + expert_list[e].n;
        for (int32_t i = 0; i < expert_list[e].n; ++i) {
            const int32_t pair = expert_list[e].v[i];
            const int32_t slot = exp_off[e] + i;
            const int32_t row = send_off[e / Eloc] + pos_in_node[pair];
            pair_slot[pair] = slot;
            slot_pair[slot] = pair;
            slot_token[slot] = pair / K;
            pair_send_row[pair] = row;
            slot_send_row[slot] = row;
        }
    }

done:
    ilists_free(node_list, D);
    ilists_free(expert_list, E);
    free(pos_in_node);
    return rc;
}

/*
 * Transfer order of the level-2 descriptors (section 3.2: a descriptor list is a dense array in transfer
 * order; the paper does not say which order, this is the reading used here).  The tokens are cut into tiles
 * of tile_tokens consecutive tokens.  The list of a tile holds the rows of the expert-activation tensor that
 * its (token, expert) pairs own, in ascending row order - so the rows of one expert follow one another, in
 * ascending token order - and is padded with -1 up to tile_tokens * K entries (a last tile with fewer tokens,
 * pairs without a row).  tile_slots has ceil(T / tile_tokens) * tile_tokens * K entries.
 */
static int cmp_int32(const void *a, const void *b)
{
    const int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

int fusco_oracle_tile_order(const int32_t *pair_slot, int32_t T, int32_t K, int32_t tile_tokens, int32_t *tile_slots)
{
    if (T < 0 || K < 1 || tile_tokens < 1 || (T > 0 && (!pair_slot || !tile_slots))) return ORACLE_ERR_ARG;
    const int64_t cap = (int64_t)tile_tokens * K;
    for (int64_t t0 = 0, tile = 0; t0 < T; t0 += tile_tokens, ++tile) {
        int32_t *list = tile_slots + tile * cap;
        int64_t n = 0;
        for (int64_t t = t0; t < t0 + tile_tokens && t < T; ++t)
            for (int32_t j = 0; j < K; ++j)
                if (pair_slot[t * K + j] >= 0) list[n++] = pair_slot[t * K + j];
        qsort(list, (size_t)n, sizeof(int32_t), cmp_int32);
        for (; n < cap; ++n) list[n] = -1;
    }
    return ORACLE_OK;
}

/*
 * Dispatch, hop by hop as the planner describes it: level 1 moves one row per (token, device)
 * into the device's receive tensor, level 2 moves every (t, e) pair from there to its row of the
 * expert-activation tensor.  Rows are opaque bytes.  send_buf has U = send_off[D] rows,
 * expert_buf has P rows.  An optional second plane (aux, e.g. per-block scales) follows the same
 * descriptors; pass aux_row_bytes = 0 to skip it.
 */
int fusco_oracle_dispatch(const uint8_t *x, int64_t row_bytes,
                          const uint8_t *x_aux, int64_t aux_row_bytes,
                          int32_t U, int32_t P,
                          const int32_t *send_src, const int32_t *slot_send_row,
                          uint8_t *send_buf, uint8_t *send_aux,
                          uint8_t *expert_buf, uint8_t *expert_aux)
{
    if (!x || !send_src || !slot_send_row || !send_buf || !expert_buf || row_bytes <= 0)
        return ORACLE_ERR_ARG;
    if (aux_row_bytes > 0 && (!x_aux || !send_aux || !expert_aux)) return ORACLE_ERR_ARG;
    for (int32_t r = 0; r < U; ++r) {
        memcpy(send_buf + (int64_t)r * row_bytes, x + (int64_t)send_src[r] * row_bytes, (size_t)row_bytes);
        if (aux_row_bytes > 0)
            memcpy(send_aux + (int64_t)r * aux_row_bytes, x_aux + (int64_t)send_src[r] * aux_row_bytes,
                   (size_t)aux_row_bytes);
    }
    for (int32_t s = 0; s < P; ++s) {
        memcpy(expert_buf + (int64_t)s * row_bytes, send_buf + (int64_t)slot_send_row[s] * row_bytes,
               (size_t)row_bytes);
        if (aux_row_bytes > 0)
            memcpy(expert_aux + (int64_t)s * aux_row_bytes,
                   send_aux + (int64_t)slot_send_row[s] * aux_row_bytes, (size_t)aux_row_bytes);
    }
    return ORACLE_OK;
}

/*
 * Dispatch for a list of expert-activation rows only (for checks at sizes where the whole tensor is
 * too large to build on the host): out row i is the payload of row slots[i], reached hop by hop as
 * in fusco_oracle_dispatch (token of the send row that the slot's level-2 send descriptor names).
 */
int fusco_oracle_dispatch_rows(const uint8_t *x, int64_t row_bytes, int32_t P,
                               const int32_t *send_src, const int32_t *slot_send_row,
                               const int32_t *slots, int32_t n_slots, uint8_t *out)
{
    if (!x || !send_src || !slot_send_row || !slots || !out || row_bytes <= 0) return ORACLE_ERR_ARG;
    for (int32_t i = 0; i < n_slots; ++i) {
        const int32_t s = slots[i];
        if (s < 0 || s >= P) return ORACLE_ERR_ARG;
        const int32_t t = send_src[slot_send_row[s]];
        memcpy(out + (int64_t)i * row_bytes, x + (int64_t)t * row_bytes, (size_t)row_bytes);
    }
    return ORACLE_OK;
}

static float bf16_to_float(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* round a float to bfloat16, ties to even; NaN stays a quiet NaN */
static uint16_t float_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
    const uint32_t lower = u & 0xFFFFu;
    uint32_t upper = u >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u))) upper += 1u;
    return (uint16_t)upper;
}

static float y_at(const void *y, int y_dtype, int64_t i)
{
    return y_dtype == ORACLE_BF16 ? bf16_to_float(((const uint16_t *)y)[i]) : ((const float *)y)[i];
}

/*
 * Combine in double precision: out[t][c] = sum_j w[t][j] * y[pair_slot[t][j]][c].
 * If tokens != NULL only the n_tokens listed tokens are computed and out has n_tokens rows
 * (row i belongs to tokens[i]); otherwise all T tokens are computed.
 */
int fusco_oracle_combine_f64(const void *y, int y_dtype, const float *w, const int32_t *pair_slot,
                             int32_t T, int32_t K, int32_t H,
                             const int32_t *tokens, int32_t n_tokens, double *out)
{
    if (!y || !w || !pair_slot || !out || K <= 0 || H <= 0) return ORACLE_ERR_ARG;
    if (y_dtype != ORACLE_BF16 && y_dtype != ORACLE_F32) return ORACLE_ERR_ARG;
    const int32_t rows = tokens ? n_tokens : T;
    for (int32_t i = 0; i < rows; ++i) {
        const int32_t t = tokens ? tokens[i] : i;
        if (t < 0 || t >= T) return ORACLE_ERR_ARG;
        for (int32_t c = 0; c < H; ++c) {
            double acc = 0.0;
            for (int32_t j = 0; j < K; ++j) {
                const int64_t s = pair_slot[(int64_t)t * K + j];
                acc += (double)w[(int64_t)t * K + j] * (double)y_at(y, y_dtype, s * H + c);
            }
            out[(int64_t)i * H + c] = acc;
        }
    }
    return ORACLE_OK;
}

/*
 * Combine in the precision the method is specified in: single-precision accumulate, one fused
 * multiply-add per term in the order j = 0..K-1 starting from +0, and a single final rounding
 * to bfloat16 (nearest even) for bfloat16 outputs.  Either output pointer may be NULL.
 */
int fusco_oracle_combine_f32(const void *y, int y_dtype, const float *w, const int32_t *pair_slot,
                             int32_t T, int32_t K, int32_t H,
                             const int32_t *tokens, int32_t n_tokens,
                             float *out_f32, uint16_t *out_bf16)
{
    if (!y || !w || !pair_slot || K <= 0 || H <= 0) return ORACLE_ERR_ARG;
    if (y_dtype != ORACLE_BF16 && y_dtype != ORACLE_F32) return ORACLE_ERR_ARG;
    const int32_t rows = tokens ? n_tokens : T;
    for (int32_t i = 0; i < rows; ++i) {
        const int32_t t = tokens ? tokens[i] : i;
        if (t < 0 || t >= T) return ORACLE_ERR_ARG;
        for (int32_t c = 0; c < H; ++c) {
            float acc = 0.0f;
            for (int32_t j = 0; j < K; ++j) {
                const int64_t s = pair_slot[(int64_t)t * K + j];
                acc = fmaf(w[(int64_t)t * K + j], y_at(y, y_dtype, s * H + c), acc);
            }
            if (out_f32) out_f32[(int64_t)i * H + c] = acc;
            if (out_bf16) out_bf16[(int64_t)i * H + c] = float_to_bf16(acc);
        }
    }
    return ORACLE_OK;
}

/* sum_j |w[t][j] * y[pair_slot[t][j]][c]| in double: the scale the combine tolerance is relative to */
int fusco_oracle_combine_abs_f64(const void *y, int y_dtype, const float *w, const int32_t *pair_slot,
                                 int32_t T, int32_t K, int32_t H,
                                 const int32_t *tokens, int32_t n_tokens, double *out)
{
    if (!y || !w || !pair_slot || !out || K <= 0 || H <= 0) return ORACLE_ERR_ARG;
    if (y_dtype != ORACLE_BF16 && y_dtype != ORACLE_F32) return ORACLE_ERR_ARG;
    const int32_t rows = tokens ? n_tokens : T;
    for (int32_t i = 0; i < rows; ++i) {
        const int32_t t = tokens ? tokens[i] : i;
        if (t < 0 || t >= T) return ORACLE_ERR_ARG;
        for (int32_t c = 0; c < H; ++c) {
            double acc = 0.0;
            for (int32_t j = 0; j < K; ++j) {
                const int64_t s = pair_slot[(int64_t)t * K + j];
                acc += fabs((double)w[(int64_t)t * K + j] * (double)y_at(y, y_dtype, s * H + c));
            }
            out[(int64_t)i * H + c] = acc;
        }
    }
    return ORACLE_OK;
}

/*
 * Combine along the two descriptor levels in reverse (the mirror of the two-hop
 * dispatch; the paper gives no arithmetic for it, this is the reading used here):
 *   level 2 reversed: every send row r = (token t, device d) receives the partial sum of the
 *     token's entries on that device, partial[r] = sum_{j : dev(A[t][j]) = d} w[t][j] * y[slot(t,j)],
 *     one fused multiply-add per term in ascending j starting from +0 (single precision);
 *   level 1 reversed: out[t] = sum of the token's partial rows, plain single-precision additions
 *     starting from +0 in the order in which the devices first appear among the token's entries.
 * Only the association of the sum differs from fusco_oracle_combine_f32.
 * partial (optional, [U][H] floats) receives the level-2 result for all send rows when tokens == NULL.
 */
int fusco_oracle_combine_two_hop_f32(const void *y, int y_dtype, const float *w, const int32_t *pair_slot,
                                     const int32_t *pair_send_row, const uint8_t *pair_first,
                                     int32_t T, int32_t K, int32_t H,
                                     const int32_t *tokens, int32_t n_tokens,
                                     float *partial, float *out_f32, uint16_t *out_bf16)
{
    if (!y || !w || !pair_slot || !pair_send_row || !pair_first || K <= 0 || H <= 0) return ORACLE_ERR_ARG;
    if (y_dtype != ORACLE_BF16 && y_dtype != ORACLE_F32) return ORACLE_ERR_ARG;
    if (partial && tokens) return ORACLE_ERR_ARG;
    const int32_t rows = tokens ? n_tokens : T;
    float *part = (float *)malloc((size_t)K * sizeof(float));   /* partial sums of one token, one column */
    if (!part) return ORACLE_ERR_MEM;
    for (int32_t i = 0; i < rows; ++i) {
        const int32_t t = tokens ? tokens[i] : i;
        if (t < 0 || t >= T) { free(part); return ORACLE_ERR_ARG; }
        const int64_t p0 = (int64_t)t * K;
        for (int32_t c = 0; c < H; ++c) {
            /* level 2 reversed: one partial per first appearance f, over the entries that share its send row */
            for (int32_t f = 0; f < K; ++f) {
                if (!pair_first[p0 + f]) continue;
                float acc = 0.0f;
                for (int32_t j = 0; j < K; ++j)
                    if (pair_send_row[p0 + j] == pair_send_row[p0 + f])
                        acc = fmaf(w[p0 + j], y_at(y, y_dtype, (int64_t)pair_slot[p0 + j] * H + c), acc);
                part[f] = acc;
                if (partial) partial[(int64_t)pair_send_row[p0 + f] * H + c] = acc;
            }
            /* level 1 reversed */
            float acc = 0.0f;
            for (int32_t f = 0; f < K; ++f)
                if (pair_first[p0 + f]) acc = acc + part[f];
            if (out_f32) out_f32[(int64_t)i * H + c] = acc;
            if (out_bf16) out_bf16[(int64_t)i * H + c] = float_to_bf16(acc);
        }
    }
    free(part);
    return ORACLE_OK;
}

/*
 * Segment-descriptor transfer (section 3.2, the paragraph on segment descriptors): a payload is a sequence of n logical segments; segment i is size[i] bytes long and
 * lies at src_off[i] in the sender's memory and at dst_off[i] in the receiver's.  The descriptor
 * lists are dense arrays in transfer order and map one to one.  A NULL offset list means that side
 * is the contiguous stream itself (segment i starts at the cumulative size of the segments before
 * it), which is how segments are bundled into slices for the network.
 * slice_fill (optional, with slice_bytes > 0): bytes of the contiguous stream that fall into every
 * slice of slice_bytes, i.e. what a consumer waits for before it takes the slice.
 */
int fusco_oracle_segments_copy(const uint8_t *src, const uint64_t *src_off, uint8_t *dst, const uint64_t *dst_off,
                               const uint64_t *size, int64_t n, uint64_t slice_bytes, uint32_t *slice_fill)
{
    if (!src || !dst || !size || n < 0) return ORACLE_ERR_ARG;
    uint64_t cum = 0;
    for (int64_t i = 0; i < n; ++i) {
        const uint64_t so = src_off ? src_off[i] : cum;
        const uint64_t dofs = dst_off ? dst_off[i] : cum;
        memcpy(dst + dofs, src + so, (size_t)size[i]);
        cum += size[i];
    }
    if (slice_fill && slice_bytes > 0) {
        const uint64_t slices = (cum + slice_bytes - 1) / slice_bytes;
        for (uint64_t s = 0; s < slices; ++s) {
            const uint64_t left = cum - s * slice_bytes;
            slice_fill[s] = (uint32_t)(left < slice_bytes ? left : slice_bytes);
        }
    }
    return ORACLE_OK;
}
