// Mover kernels: fused gather-pack (dispatch), weighted combine, their two-hop and staged variants.
#ifndef FUSCO_CSRC_MOVERS_H
#define FUSCO_CSRC_MOVERS_H

#include "common.h"
#include "planner.h"

namespace {

// ------------------------------------------------------------------------------------------
// Movers.  A row is fetched or written whole by the waves of one workgroup within a short time.
// Measured on MI355X at 14 KiB rows: scattered row reads come close to the streaming read rate
// (6.4-6.6 of 7.2 TB/s), scattered row writes do not (5.2-5.4 of 6.9 TB/s), and what the write
// rate depends on is which XCD writes which neighbouring addresses.  Combine therefore walks the
// tokens (its scattered side is the reads), and dispatch writes in the planner's transfer order
// where it can (dispatch_tiled_kernel) and walks the tokens otherwise (dispatch_kernel).
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ u32x4 load16_stream(const u32x4 *p) { return __builtin_nontemporal_load(p); }

// 16-byte / 8-byte write-through stores at device scope (sc1): the data leaves the L2 of the XCD for
// memory instead of lingering there.  Used for the token-ordered output of combine, which is never
// read again by this kernel.
// The s_nop supplies the wait states gfx9 needs between a store of more than 8 bytes and a
// following VALU write to its data registers; the compiler adds them for its own stores but
// cannot see into this statement.
__device__ __forceinline__ void store16_through(u32x4 *p, u32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void store8_through(u32x2 *p, u32x2 v)
{
    asm volatile("global_store_dwordx2 %0, %1, off sc1\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
}
// Write-through and non-temporal together (sc1 nt): the tiled dispatch's destination rows.  Measured against
// the plain non-temporal store at 8192 tokens x 8 rows of 14 KiB: 169 us instead of 174 us in a loop over the same
// buffers, 160 us instead of 174 us after other traffic has gone through the memory-side cache, never slower.
__device__ __forceinline__ void store16_through_stream(u32x4 *p, u32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
}
// The same at system scope (sc0 sc1): for data that another agent may read once a flag says so.
__device__ __forceinline__ void store16_system(u32x4 *p, u32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
}

// Dispatch: the row is held in registers between the single read and the k (+ wire) writes.
// Slot lookups depend only on blockIdx, so they are scalar loads.
struct DispatchArgs {
    const u32x4 *x, *x_aux;
    u32x4 *expert_buf, *expert_aux, *send_buf, *send_aux;
    const int32_t *pair_slot, *pair_send_row;
    const uint8_t *pair_first;
    const int32_t *slot_token, *tile_slots;   // tiled mode: transfer order of every tile
    int32_t tile_cap;                         // entries per tile in tile_slots
    int32_t tile_tokens;                      // tokens per tile
    int32_t N;                                // tokens in all
    int32_t segs;                             // workgroups per row: a row longer than a workgroup covers is cut into columns
    int32_t seg_chunks;                       // 16-byte chunks per column segment (the last one may be shorter)
    int32_t k;
    int32_t C, Ca;   // 16-byte chunks per row in the main and in the aux plane
    int32_t write_expert, write_wire;
};

constexpr int kXcds = 8;                                  // accelerator complexes of an MI355X
constexpr int kTiledMinTiles = 2 * kXcds;                 // fewer tiles would leave XCDs idle
constexpr size_t kTiledMaxTileBytes = (size_t)3840 << 10; // source rows of one tile must fit a 4 MB L2
constexpr size_t kSourceChunkBytes = (size_t)128 << 20;   // source rows of one chunk: half the 256 MB memory-side cache
constexpr size_t kCacheBytes = (size_t)256 << 20;         // the memory-side cache
constexpr size_t kTiledShortRowBytes = 8192;              // rows below this are tiled only with a small source tensor
constexpr size_t kResidentSourceBytes = (size_t)116 << 20; // largest source tensor that stays in that cache next to an output of its size

// Loads and stores of the token walk (MODE of dispatch_kernel: bit 0 cached loads, bit 1 non-temporal stores).
// Non-temporal stores go past the memory-side cache (a read that follows such a write runs at the cold rate,
// 5.7 TB/s for 256 MB, instead of 4.2 TB/s on rows that sit dirty in that cache); plain stores leave the rows
// there, which is what a reader of a tensor of up to 256 MB wants.  With non-temporal stores a source tensor
// that fits that cache is read with plain cached loads and stays there from one call to the next, since
// nothing the kernel writes displaces it (8192 tokens x 8 rows of 14 KiB: 187 us instead of 208 us; non-temporal
// loads together with non-temporal stores take 215 us there); a larger one is read with non-temporal loads
// (32768 tokens x 2 rows of 8 KiB: 138 us, against 168 us with cached loads).  walk_mode in fusco.hip chooses.
template <bool STREAM>
__device__ __forceinline__ void put16(u32x4 *p, u32x4 v)
{
    if constexpr (STREAM) __builtin_nontemporal_store(v, p);
    else *p = v;
}

template <int CPT, int MODE = 0>   // MODE bit 0: cached loads, bit 1: non-temporal stores
__global__ __launch_bounds__(256) void dispatch_kernel(DispatchArgs a)
{
    // workgroup = (token, column segment), segments of one row next to each other in launch order, so that a
    // row longer than one workgroup covers is still read and written as a whole within a short time
    const int t = blockIdx.x / (uint32_t)a.segs, seg = blockIdx.x - (uint32_t)t * a.segs;
    const int Ct = a.C + a.Ca;
    const int c_end = min(Ct, (seg + 1) * a.seg_chunks);   // this segment: chunks [seg * seg_chunks, c_end)
    const int c0 = seg * a.seg_chunks + threadIdx.x;
    u32x4 v[CPT];
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        const int c = c0 + i * blockDim.x;
        const u32x4 *src = c < a.C ? a.x + (size_t)t * a.C + c : a.x_aux + (size_t)t * a.Ca + (c - a.C);
        if (c < c_end) v[i] = (MODE & 1) ? *src : load16_stream(src);
    }
    const int32_t *slots = a.pair_slot + (size_t)t * a.k;
    if (a.write_expert) {
        for (int j = 0; j < a.k; ++j) {
            const int slot = slots[j];
            if (slot < 0) continue;
#pragma unroll
            for (int i = 0; i < CPT; ++i) {
                const int c = c0 + i * blockDim.x;
                if (c >= c_end) continue;
                if (c < a.C) put16<(MODE & 2) != 0>(a.expert_buf + (size_t)slot * a.C + c, v[i]);
                else put16<(MODE & 2) != 0>(a.expert_aux + (size_t)slot * a.Ca + (c - a.C), v[i]);
            }
        }
    }
    if (a.write_wire) {
        const int32_t *rows = a.pair_send_row + (size_t)t * a.k;
        const uint8_t *first = a.pair_first + (size_t)t * a.k;
        for (int j = 0; j < a.k; ++j) {
            if (!first[j]) continue;
            const int row = rows[j];
#pragma unroll
            for (int i = 0; i < CPT; ++i) {
                const int c = c0 + i * blockDim.x;
                if (c >= c_end) continue;
                if (c < a.C) put16<(MODE & 2) != 0>(a.send_buf + (size_t)row * a.C + c, v[i]);
                else put16<(MODE & 2) != 0>(a.send_aux + (size_t)row * a.Ca + (c - a.C), v[i]);
            }
        }
    }
}

// Dispatch in transfer order (the tile_slots list of the planner): one workgroup per destination row.  The
// hardware hands workgroups to the 8 XCDs in turn, so workgroup b = 8 i + x runs on XCD x; it takes entry
// i mod cap of tile x + 8 (i / cap).  An XCD therefore works through whole tiles, one after the other, and
// inside a tile it writes expert by expert: the rows of one expert are neighbours in memory, written by one
// XCD within a short time.  Every source row is needed k times by the tile; it comes from memory once and
// from the XCD's L2 afterwards (plain cached loads; a tile's source rows, or the column segment of them that
// a pass moves, fit the L2).  The rows are written with non-temporal write-through stores
// (store16_through_stream): they do not displace the source rows from the L2 - the fabric counters show
// every source row fetched 1.03 times, against 1.4 times with plain non-temporal stores - and they go past
// the memory-side cache, which the next reader of memory would otherwise have to clean first and which so
// keeps a source tensor that fits it from one call to the next.  The reads are hidden completely: the kernel
// runs at the rate of its write pattern, and that rate goes up when fewer rows are being written at a time.
// The launch therefore caps the workgroups per compute unit for long rows (tiled_workgroups_per_cu: dynamic LDS
// that the kernel does not use).  Measured on MI355X at 8192 tokens x 8 rows of 14 KiB, source tensor in the
// memory-side cache / cold in memory: 8 workgroups per compute unit 164 / 203 us, 5 workgroups 151 / 222 us,
// 5 workgroups with PULL 157 / 178 us.  The token walk takes 205 us with non-temporal loads and plain stores
// and 187 us with cached loads and non-temporal stores.
// PULL: the first tile_tokens workgroups of a pass also read one source row of the tile each (see below).
// AUX: the second plane exists.  A chunk's source and destination are picked by address selection, not by
// branching, so that the loads of a thread are issued back to back (a branch per chunk costs 3 % here).
// The launch covers the tiles [tile_base, tile_base + tiles_here).
template <int CPT, bool AUX, bool PULL>
__global__ __launch_bounds__(256) void dispatch_tiled_kernel(DispatchArgs a, uint32_t tile_base, uint32_t tiles_here)
{
    // a tile is worked through a.segs times, once per column segment of the rows (one pass for rows that a
    // workgroup covers): the L2 then only has to hold that segment of the tile's source rows
    const uint32_t b = blockIdx.x, x = b & (kXcds - 1), i = b / kXcds;
    const uint32_t per_tile = (uint32_t)a.tile_cap * (uint32_t)a.segs;
    const uint32_t round = i / per_tile, w = i - round * per_tile;
    const uint32_t pass = w / (uint32_t)a.tile_cap, r = w - pass * (uint32_t)a.tile_cap;
    const uint32_t local = x + kXcds * round;
    if (local >= tiles_here) return;
    const uint32_t tile = tile_base + local;
    const int slot = a.tile_slots[(size_t)tile * a.tile_cap + r];
    const int Ct = AUX ? a.C + a.Ca : a.C;
    // PULL: the first tile_tokens workgroups of a pass also read one source row of the tile each (the segment
    // of it that this pass moves) and drop it.  All of the tile's source rows are then on their way to the L2
    // while the tile's first entries are written, instead of every first use of a row waiting for memory in its
    // own workgroup: with few workgroups per compute unit that wait is what a cold source tensor costs.
    const int tp = (int)(tile * (uint32_t)a.tile_tokens + r);
    const bool pull = PULL && r < (uint32_t)a.tile_tokens && tp < a.N;
    u32x4 p[CPT];
    const uint32_t pseg = a.segs > 1 ? (pass + (uint32_t)tp) % (uint32_t)a.segs : 0u;
    const int p_end = min(Ct, (int)(pseg + 1) * a.seg_chunks), p0 = pseg * a.seg_chunks + threadIdx.x;
    if (pull) {
#pragma unroll
        for (int q = 0; q < CPT; ++q) {
            const int c = p0 + q * blockDim.x;
            const u32x4 *src = a.x + (size_t)tp * a.C + c;
            if (AUX && c >= a.C) src = a.x_aux + (size_t)tp * a.Ca + (c - a.C);
            if (c < p_end) p[q] = *src;
        }
    }
    if (slot >= 0) {
        const int t = a.slot_token[slot];
        // which segment a pass moves rotates with the token: the segments in use during a pass then lie at different
        // offsets in their rows, and rows whose size is a power of two do not all fall on the same sets of the L2
        const uint32_t seg = a.segs > 1 ? (pass + (uint32_t)t) % (uint32_t)a.segs : 0u;
        const int c_end = min(Ct, (int)(seg + 1) * a.seg_chunks);   // this segment: chunks [seg * seg_chunks, c_end)
        const int c0 = seg * a.seg_chunks + threadIdx.x;
        u32x4 v[CPT];
#pragma unroll
        for (int q = 0; q < CPT; ++q) {
            const int c = c0 + q * blockDim.x;
            const u32x4 *src = a.x + (size_t)t * a.C + c;
            if (AUX && c >= a.C) src = a.x_aux + (size_t)t * a.Ca + (c - a.C);
            if (c < c_end) v[q] = *src;
        }
#pragma unroll
        for (int q = 0; q < CPT; ++q) {
            const int c = c0 + q * blockDim.x;
            u32x4 *dst = a.expert_buf + (size_t)slot * a.C + c;
            if (AUX && c >= a.C) dst = a.expert_aux + (size_t)slot * a.Ca + (c - a.C);
            if (c < c_end) store16_through_stream(dst, v[q]);
        }
    }
    if (pull) {
#pragma unroll
        for (int q = 0; q < CPT; ++q)
            if (p0 + q * (int)blockDim.x < p_end) asm volatile("" ::"v"(p[q]));   // the value is not used: only the read matters
    }
}

// Reads n 16-byte units once, 4 KiB per workgroup in address order, and drops them: afterwards they sit in the
// memory-side cache.  The tiled dispatch of a source tensor larger than half that cache runs it over the source rows
// of the next chunk of tiles, so that they reach memory as one sequential burst of reads, with no writes in
// flight, instead of trickling out between the writes (measured at 32 Ki tokens of 14 KiB, chunks of 32 tiles:
// 760 us instead of 824 us; as part of the tiled kernel's own launch the reads did not help).
__global__ __launch_bounds__(256) void touch_kernel(const u32x4 *src, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const u32x4 v = src[i];
    asm volatile("" ::"v"(v));   // the value is not used: only the read matters
}

// Planner and dispatch in one launch for inputs of a single planner tile (decode-sized batches, where
// three dependent launches cost more than the work): one workgroup per token, every workgroup works out the
// whole plan in its own LDS (a few microseconds, all in parallel), workgroup 0 writes the descriptor
// arrays, and each workgroup then moves its token's row to the slots it has just computed.  The row is
// requested before the planning starts, so that its latency hides behind it.
constexpr int kFusedPreload = 4;   // 16-byte chunks per thread held in registers across the planning

template <int R>
__global__ __launch_bounds__(kPlanThreads) void plan_dispatch_kernel(PlanArgs a, DispatchArgs m)
{
    __shared__ PlaceLds<R> s;
    const int tid = threadIdx.x;
    const int t = blockIdx.x;   // the grid has max(N, 1) workgroups
    const int Ct = m.C + m.Ca;
    u32x4 v[kFusedPreload];
    if (t < a.N) {
#pragma unroll
        for (int i = 0; i < kFusedPreload; ++i) {
            const int c = tid + i * kPlanThreads;
            if (c < m.C) v[i] = load16_stream(m.x + (size_t)t * m.C + c);
            else if (c < Ct) v[i] = load16_stream(m.x_aux + (size_t)t * m.Ca + (c - m.C));
        }
    }
    place_tile<true, R>(s, a, 0, blockIdx.x == 0);
    __syncthreads();
    if (t >= a.N) return;
    const int *slots = s.tile_slot + t * a.k;
    for (int j = 0; j < a.k; ++j) {
        const int slot = slots[j];
        if (slot < 0) continue;
#pragma unroll
        for (int i = 0; i < kFusedPreload; ++i) {
            const int c = tid + i * kPlanThreads;
            if (c < m.C) m.expert_buf[(size_t)slot * m.C + c] = v[i];
            else if (c < Ct) m.expert_aux[(size_t)slot * m.Ca + (c - m.C)] = v[i];
        }
    }
    // rows longer than the preloaded part
    for (int c = tid + kFusedPreload * kPlanThreads; c < Ct; c += kPlanThreads) {
        const u32x4 u = c < m.C ? load16_stream(m.x + (size_t)t * m.C + c)
                                : load16_stream(m.x_aux + (size_t)t * m.Ca + (c - m.C));
        for (int j = 0; j < a.k; ++j) {
            const int slot = slots[j];
            if (slot < 0) continue;
            if (c < m.C) m.expert_buf[(size_t)slot * m.C + c] = u;
            else m.expert_aux[(size_t)slot * m.Ca + (c - m.C)] = u;
        }
    }
}

// Combine: every thread owns CPT 16-byte chunks of the output row, pulls the matching chunks of
// the token's k rows (JU rows in flight at a time) and accumulates in fp32 with one fused
// multiply-add per term in ascending j.
struct CombineArgs {
    const u32x4 *y;
    const float *w;
    void *out;
    const int32_t *pair_slot;
    int32_t k;
    int32_t C;   // 16-byte chunks per y row
    int32_t first;   // row handled by workgroup 0; the walk goes upwards from there and wraps around
    int32_t n_rows;  // rows of the walk (tokens, or send rows in the per-send-row mode)
    int32_t segs;    // workgroups per row: the columns of a row longer than one workgroup covers
    // per-send-row mode (level 2 reversed): one workgroup per send row, only the token's entries on that row
    const int32_t *pair_send_row, *send_src, *n_rows_dev;
};

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }

// fp32 -> bfloat16 bits, round to nearest even, NaN kept quiet
__device__ __forceinline__ uint32_t to_bf16(float f)
{
    const uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

template <bool Y_BF16, bool OUT_BF16, int CPT, int JU, bool PER_SEND_ROW = false>
__global__ __launch_bounds__(1024) void combine_kernel(CombineArgs a)
{
    constexpr int EPC = Y_BF16 ? 8 : 4;   // elements per 16-byte chunk of y
    // The walk starts at row a.first and wraps: when combine follows dispatch, the rows of the last
    // tokens are still in the memory-side cache, and reading them first, oldest first, finds them
    // there before the walk's own traffic pushes them out (see combine_first_row).
    // workgroup = (row, column segment), the segments of one row next to each other in launch order
    const int walk = blockIdx.x / (uint32_t)a.segs, seg = blockIdx.x - (uint32_t)walk * a.segs;
    int r = a.first + walk;   // token, or send row in the per-send-row mode
    if (r >= a.n_rows) r -= a.n_rows;
    int t = r;
    if constexpr (PER_SEND_ROW) {
        if (r >= *a.n_rows_dev) return;
        t = a.send_src[r];
    }
    const int c0 = seg * (blockDim.x * CPT) + threadIdx.x;
    const int32_t *slots = a.pair_slot + (size_t)t * a.k;
    const float *wt = a.w + (size_t)t * a.k;

    float acc[CPT][EPC];
#pragma unroll
    for (int i = 0; i < CPT; ++i)
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[i][e] = 0.0f;

    for (int j0 = 0; j0 < a.k; j0 += JU) {
        u32x4 v[JU][CPT];
        float wj[JU];
        bool on[JU];
#pragma unroll
        for (int jj = 0; jj < JU; ++jj) {
            const int j = j0 + jj;
            on[jj] = false;
            if (j < a.k) {
                const int slot = slots[j];
                wj[jj] = wt[j];
                bool take = slot >= 0;
                if constexpr (PER_SEND_ROW) take = take && a.pair_send_row[(size_t)t * a.k + j] == r;
                if (take) {
                    on[jj] = true;
#pragma unroll
                    for (int i = 0; i < CPT; ++i) {
                        const int c = c0 + i * blockDim.x;
                        if (c < a.C) v[jj][i] = load16_stream(a.y + (size_t)slot * a.C + c);
                    }
                }
            }
        }
#pragma unroll
        for (int jj = 0; jj < JU; ++jj) {
            if (!on[jj]) continue;
#pragma unroll
            for (int i = 0; i < CPT; ++i) {
                if constexpr (Y_BF16) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        acc[i][2 * q] = __builtin_fmaf(wj[jj], bf16_lo(v[jj][i][q]), acc[i][2 * q]);
                        acc[i][2 * q + 1] = __builtin_fmaf(wj[jj], bf16_hi(v[jj][i][q]), acc[i][2 * q + 1]);
                    }
                } else {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        acc[i][q] = __builtin_fmaf(wj[jj], __uint_as_float(v[jj][i][q]), acc[i][q]);
                }
            }
        }
    }

#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        const int c = c0 + i * blockDim.x;
        if (c >= a.C) continue;
        const size_t e0 = ((size_t)r * a.C + c) * EPC;   // first output element of this chunk
        if constexpr (OUT_BF16) {
            uint32_t pk[EPC / 2];
#pragma unroll
            for (int q = 0; q < EPC / 2; ++q) pk[q] = to_bf16(acc[i][2 * q]) | (to_bf16(acc[i][2 * q + 1]) << 16);
            if constexpr (Y_BF16) {
                u32x4 o = {pk[0], pk[1], pk[2], pk[3]};
                store16_through((u32x4 *)((uint16_t *)a.out + e0), o);
            } else {
                u32x2 o = {pk[0], pk[1]};
                store8_through((u32x2 *)((uint16_t *)a.out + e0), o);
            }
        } else {
#pragma unroll
            for (int h = 0; h < EPC / 4; ++h) {
                u32x4 o = {__float_as_uint(acc[i][4 * h]), __float_as_uint(acc[i][4 * h + 1]),
                           __float_as_uint(acc[i][4 * h + 2]), __float_as_uint(acc[i][4 * h + 3])};
                store16_through((u32x4 *)((float *)a.out + e0) + h, o);
            }
        }
    }
}

// Two-hop combine for k <= 8 in one pass: the token's k source chunks are loaded once, the partial
// sum of every destination device is formed (same operation order as the two-kernel path: fused
// multiply-adds in ascending j inside a device, then plain additions of the partial sums in order
// of first appearance), stored to the device's partial row, and added to the token's output.
struct TwoHopArgs {
    const u32x4 *y;
    const float *w;
    float *partial;
    void *out;
    const int32_t *pair_slot, *pair_send_row;
    const uint8_t *pair_first;
    int32_t k;
    int32_t C;   // 16-byte chunks per y row
};

template <bool Y_BF16, bool OUT_BF16>
__global__ __launch_bounds__(1024) void combine_two_hop_kernel(TwoHopArgs a)
{
    constexpr int EPC = Y_BF16 ? 8 : 4;
    constexpr int KMAX = 8;
    const int t = gridDim.x - 1 - blockIdx.x;
    const int c = blockIdx.y * blockDim.x + threadIdx.x;
    if (c >= a.C) return;
    const int32_t *slots = a.pair_slot + (size_t)t * a.k;
    const int32_t *rows = a.pair_send_row + (size_t)t * a.k;
    const uint8_t *first = a.pair_first + (size_t)t * a.k;
    const float *wt = a.w + (size_t)t * a.k;

    u32x4 v[KMAX];
    int row[KMAX];
    float wj[KMAX];
    bool on[KMAX], lead[KMAX];
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
        on[j] = false;
        lead[j] = false;
        row[j] = -1;
        if (j < a.k) {
            const int slot = slots[j];
            row[j] = rows[j];
            wj[j] = wt[j];
            lead[j] = first[j];
            if (slot >= 0) {
                on[j] = true;
                v[j] = load16_stream(a.y + (size_t)slot * a.C + c);
            }
        }
    }
    float total[EPC];
#pragma unroll
    for (int e = 0; e < EPC; ++e) total[e] = 0.0f;
#pragma unroll
    for (int f = 0; f < KMAX; ++f) {
        if (!lead[f]) continue;
        float acc[EPC];
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[e] = 0.0f;
#pragma unroll
        for (int j = 0; j < KMAX; ++j) {
            if (!on[j] || row[j] != row[f]) continue;
            if constexpr (Y_BF16) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    acc[2 * q] = __builtin_fmaf(wj[j], bf16_lo(v[j][q]), acc[2 * q]);
                    acc[2 * q + 1] = __builtin_fmaf(wj[j], bf16_hi(v[j][q]), acc[2 * q + 1]);
                }
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[q] = __builtin_fmaf(wj[j], __uint_as_float(v[j][q]), acc[q]);
            }
        }
        u32x4 *prow = (u32x4 *)(a.partial + ((size_t)row[f] * a.C + c) * EPC);
#pragma unroll
        for (int h = 0; h < EPC / 4; ++h) {
            const u32x4 o = {__float_as_uint(acc[4 * h]), __float_as_uint(acc[4 * h + 1]),
                             __float_as_uint(acc[4 * h + 2]), __float_as_uint(acc[4 * h + 3])};
            prow[h] = o;
        }
#pragma unroll
        for (int e = 0; e < EPC; ++e) total[e] = total[e] + acc[e];
    }
    const size_t e0 = ((size_t)t * a.C + c) * EPC;
    if constexpr (OUT_BF16) {
        uint32_t pk[EPC / 2];
#pragma unroll
        for (int q = 0; q < EPC / 2; ++q) pk[q] = to_bf16(total[2 * q]) | (to_bf16(total[2 * q + 1]) << 16);
        if constexpr (Y_BF16) {
            const u32x4 o = {pk[0], pk[1], pk[2], pk[3]};
            store16_through((u32x4 *)((uint16_t *)a.out + e0), o);
        } else {
            const u32x2 o = {pk[0], pk[1]};
            store8_through((u32x2 *)((uint16_t *)a.out + e0), o);
        }
    } else {
#pragma unroll
        for (int h = 0; h < EPC / 4; ++h) {
            const u32x4 o = {__float_as_uint(total[4 * h]), __float_as_uint(total[4 * h + 1]),
                             __float_as_uint(total[4 * h + 2]), __float_as_uint(total[4 * h + 3])};
            store16_through((u32x4 *)((float *)a.out + e0) + h, o);
        }
    }
}

// Level 1 reversed: out[t] = sum of the token's partial rows (fp32, one per destination device),
// plain additions from +0 in the order in which the devices first appear among the token's entries.
struct SumPartialsArgs {
    const u32x4 *partial;   // [send rows, C] chunks of 4 floats
    void *out;
    const int32_t *pair_send_row;
    const uint8_t *pair_first;
    int32_t k;
    int32_t C;              // 16-byte chunks (4 floats) per partial row
};

template <bool OUT_BF16>
__global__ __launch_bounds__(1024) void sum_partials_kernel(SumPartialsArgs a)
{
    const int t = gridDim.x - 1 - blockIdx.x;
    const int c = blockIdx.y * blockDim.x + threadIdx.x;
    if (c >= a.C) return;
    const int32_t *rows = a.pair_send_row + (size_t)t * a.k;
    const uint8_t *first = a.pair_first + (size_t)t * a.k;
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int j0 = 0; j0 < a.k; j0 += 8) {
        u32x4 v[8];
        bool on[8];
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            const int j = j0 + jj;
            on[jj] = j < a.k && first[j];
            if (on[jj]) v[jj] = load16_stream(a.partial + (size_t)rows[j] * a.C + c);
        }
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            if (!on[jj]) continue;
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] = acc[q] + __uint_as_float(v[jj][q]);
        }
    }
    const size_t e0 = ((size_t)t * a.C + c) * 4;
    if constexpr (OUT_BF16) {
        u32x2 o = {to_bf16(acc[0]) | (to_bf16(acc[1]) << 16), to_bf16(acc[2]) | (to_bf16(acc[3]) << 16)};
        store8_through((u32x2 *)((uint16_t *)a.out + e0), o);
    } else {
        u32x4 o = {__float_as_uint(acc[0]), __float_as_uint(acc[1]), __float_as_uint(acc[2]), __float_as_uint(acc[3])};
        store16_through((u32x4 *)((float *)a.out + e0), o);
    }
}

// Row gather in destination order: dst[r] = src[idx2 ? idx2[idx1[r]] : idx1[r]] for r < n_rows, one
// workgroup column per destination row.  n_rows_dev, when set, is a device-resident row count that
// caps n_rows (data-dependent lengths such as U).  Used by the two-hop dispatch (second hop) and by
// the disaggregated baseline, whose every stage is such a pass over the whole buffer.
struct GatherArgs {
    const u32x4 *src;
    u32x4 *dst;
    const int32_t *idx1, *idx2;
    const int32_t *n_rows_dev;
    int32_t C;   // 16-byte chunks per row
};

template <int CPT, bool STREAM_LOAD>
__global__ __launch_bounds__(256) void gather_rows_kernel(GatherArgs a)
{
    const int r = blockIdx.x;
    if (a.n_rows_dev && r >= *a.n_rows_dev) return;
    int q = a.idx1[r];
    if (q >= 0 && a.idx2) q = a.idx2[q];
    if (q < 0) return;
    const int c0 = blockIdx.y * (blockDim.x * CPT) + threadIdx.x;
    u32x4 v[CPT];
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        const int c = c0 + i * blockDim.x;
        if (c < a.C) v[i] = STREAM_LOAD ? load16_stream(a.src + (size_t)q * a.C + c) : a.src[(size_t)q * a.C + c];
    }
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        const int c = c0 + i * blockDim.x;
        if (c < a.C) a.dst[(size_t)r * a.C + c] = v[i];
    }
}

// dev[p] = device of expert A[p] (or -1 for an id outside [0, E)): the key of the rank-major order
__global__ __launch_bounds__(256) void expert_to_device_kernel(int32_t *dev, const int32_t *A, int64_t n, int E, int Eloc)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n) return;
    const int e = A[p];
    dev[p] = (unsigned)e < (unsigned)E ? e / Eloc : -1;
}

}   // namespace

#endif
