// MoE token shuffle with fused layout transformation for MI355X (gfx950, wave64).
//
// Three groups of kernels behind the C boundary declared in fusco.h:
//   planner  - token-expert matrix -> two-level layout descriptor (paper section 3.3)
//   dispatch - read every token row once, store it to all of its final rows (section 3.2)
//   combine  - per token, gather its k expert-output rows, weighted fp32 sum, one row out
// The path is pure data movement (no dense contraction), so there is no MFMA here: the movers
// are built around 16-byte coalesced global accesses, the planner around LDS counters and
// wave64 ballots.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <stdint.h>
#include <stdlib.h>

#include "fusco.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;
constexpr int kPlanThreads = 1024;                      // 16 waves per planner workgroup
constexpr int kPlanWaves = kPlanThreads / kWave;
constexpr int kTilePairs = 1024;                        // (token, expert) pairs per planner tile
constexpr int kRounds = kTilePairs / kPlanThreads;      // 64-pair rounds per wave
constexpr int kWaveChunk = kTilePairs / kPlanWaves;     // consecutive pairs owned by one wave
constexpr int kMaxBins = FUSCO_MAX_E;
constexpr size_t kMaxRowChunks = FUSCO_MAX_ROW_BYTES / 16;

static_assert(kTilePairs >= FUSCO_MAX_K, "a tile must hold at least one token");
static_assert(kMaxBins <= kPlanThreads, "the planner gives every bin a thread");

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

bool sizes_ok(int32_t N, int32_t k, int32_t E, int32_t D)
{
    if (N < 0 || k < 1 || k > FUSCO_MAX_K || E < 1 || E > FUSCO_MAX_E || D < 1 || D > E) return false;
    if (E % D != 0) return false;
    if ((int64_t)N * k >= ((int64_t)1 << 31)) return false;
    return true;
}

// From this many tiles on, per-tile counts are first summed over chunks of tiles (one more small launch),
// so that a placement workgroup reads about 2 * sqrt(tiles) rows of counts instead of one per tile.
constexpr int kChunkMinTiles = 320;

inline int tokens_per_tile(int k) { return kTilePairs / k; }
inline int num_tiles(int N, int k)
{
    const int tpt = tokens_per_tile(k);
    const int n = (N + tpt - 1) / tpt;
    return n < 1 ? 1 : n;
}

// tiles per chunk (a power of two near sqrt(n_tiles)), or 0 when the tiles are few enough to be read one by one
inline int chunk_tiles_for(int n_tiles)
{
    if (n_tiles < kChunkMinTiles) return 0;
    int c = 8;
    while (c * c < n_tiles) c *= 2;
    return c;
}
inline int num_chunks(int n_tiles)
{
    const int c = chunk_tiles_for(n_tiles);
    return c ? (n_tiles + c - 1) / c : 0;
}

// ------------------------------------------------------------------------------------------
// Planner
// ------------------------------------------------------------------------------------------
struct PlanArgs {
    const int32_t *A;
    int32_t N, k, E, D, Eloc;
    uint32_t k_magic, eloc_magic;   // ceil(2^20 / k), ceil(2^20 / Eloc): see div20
    int32_t tpt;      // tokens per tile
    int32_t n_tiles;
    int32_t stride;   // ints per tile in tile_hist: E expert counts, D device counts, 1 invalid count
    int32_t *tile_hist;
    int32_t chunk_tiles, n_chunks;   // 0, 0: no chunk level
    int32_t *chunk_hist;             // [n_chunks][stride]: tile_hist summed over the tiles of a chunk
    int32_t *exp_count, *exp_off, *send_count, *send_off;
    int32_t *pair_slot, *slot_pair, *slot_token, *send_src, *pair_send_row, *slot_send_row;
    uint8_t *pair_first;
    int32_t *status;
};

__device__ __forceinline__ int bits_for(int nb)
{
    int n = 0;
    while ((1 << n) < nb) ++n;
    return n;
}

// Lanes of this wave that take part and hold the same key as the calling lane.
__device__ __forceinline__ uint64_t same_key_lanes(int key, bool part, int nbits)
{
    uint64_t m = __builtin_amdgcn_ballot_w64(part);
    for (int b = 0; b < nbits; ++b) {
        const bool bit = (key >> b) & 1;
        const uint64_t bal = __builtin_amdgcn_ballot_w64(bit);
        m &= bit ? bal : ~bal;
    }
    return m;
}

// n / d for the small operands of the planner (n < 2048 with d <= 64, or n < 1024 with d <= 1024; the
// callers stay below: pair index in a tile < 1024 over k <= 64, expert id < 1024 over E / D)
// through magic = ceil(2^20 / d): the error n * (magic * d - 2^20) / (d * 2^20) stays below 1 / d.
__device__ __forceinline__ int div20(int n, uint32_t magic) { return (int)(((uint32_t)n * magic) >> 20); }

// Orders LDS traffic between the lanes of one wave (no instruction is emitted: LDS serves the
// accesses of a wave in program order, the fences only stop the compiler from moving them).
__device__ __forceinline__ void wave_lds_order()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// For the pair at tile-local index p, held by lane `lane` of a round of 64 consecutive pairs:
// the tile-local index of the first entry of the same token whose expert lives on the same device
// d (p itself if this pair is that first appearance), or -1 if d < 0.  Must be called by all lanes.
// `same` receives the lanes of the round with the same device.  tile_dev holds the device of every
// pair of the tile, row0 is the token's first pair.  Entries of the token inside this round are
// compared with ballots; only a token that straddles the round's start needs LDS reads.
__device__ __forceinline__ int first_pair_on_device(const int16_t *tile_dev, int p, int lane, int row0, int d, int dbits,
                                                    uint64_t &same)
{
    same = same_key_lanes(d, d >= 0, dbits);
    if (d < 0) return -1;
    const int base = p - lane;
    for (int q = row0; q < base; ++q)
        if (tile_dev[q] == d) return q;
    const int l0 = max(row0 - base, 0);
    const uint64_t before = same & (((uint64_t)1 << lane) - 1) & ~(((uint64_t)1 << l0) - 1);
    return before ? base + __builtin_ctzll(before) : p;
}

// Pass 1 of the multi-tile planner: per-tile counts of pairs per expert and of first
// (token, device) appearances per device.  Lanes of a wave that hold the same key are found with
// ballots and only one of them adds their number to the LDS counter, so a popular key does not
// serialise the wave.  Counts do not depend on the order of the additions.
__global__ __launch_bounds__(kPlanThreads) void plan_count_kernel(PlanArgs a)
{
    __shared__ int16_t tile_dev[kTilePairs];
    __shared__ int hist[2 * kMaxBins + 1];
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int tile = blockIdx.x;
    const int tok0 = tile * a.tpt;
    const int ntok = min(a.tpt, a.N - tok0);
    const int npairs = ntok > 0 ? ntok * a.k : 0;
    const int64_t pair0 = (int64_t)tok0 * a.k;
    const int nb = a.E + a.D;
    const int ebits = bits_for(a.E), dbits = bits_for(a.D);
    const uint64_t lt = ((uint64_t)1 << lane) - 1;

    for (int b = tid; b <= nb; b += kPlanThreads) hist[b] = 0;
    int ekey[kRounds];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = r * kPlanThreads + tid;
        int key = -1;
        bool bad = false;
        if (p < npairs) {
            const int e = a.A[pair0 + p];
            if ((unsigned)e < (unsigned)a.E) key = e;
            else bad = true;
        }
        ekey[r] = key;
        tile_dev[p] = (int16_t)(key >= 0 ? div20(key, a.eloc_magic) : -1);
        const uint64_t nbad = __builtin_amdgcn_ballot_w64(bad);
        if (r == 0) __syncthreads();   // counters are zero from here on
        if (nbad != 0 && lane == 0) atomicAdd(&hist[nb], __builtin_popcountll(nbad));
        const uint64_t m = same_key_lanes(key, key >= 0, ebits);
        if (key >= 0 && (m & lt) == 0) atomicAdd(&hist[key], __builtin_popcountll(m));
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = r * kPlanThreads + tid;
        const int d = tile_dev[p];
        uint64_t same;
        const bool first = first_pair_on_device(tile_dev, p, lane, div20(p, a.k_magic) * a.k, d, dbits, same) == p;
        const uint64_t m = same & __builtin_amdgcn_ballot_w64(first);
        if (first && (m & lt) == 0) atomicAdd(&hist[a.E + d], __builtin_popcountll(m));
    }
    __syncthreads();
    int32_t *out = a.tile_hist + (int64_t)tile * a.stride;
    for (int b = tid; b <= nb; b += kPlanThreads) out[b] = hist[b];
}

// Optional pass between counting and placing: sums the per-tile counts over chunks of consecutive
// tiles.  One workgroup per chunk; the columns are covered 1024 at a time, and where fewer columns
// than threads remain the tiles of the chunk are split over groups of threads.
__global__ __launch_bounds__(kPlanThreads) void plan_chunk_kernel(PlanArgs a)
{
    __shared__ int acc[kPlanThreads];
    const int tid = threadIdx.x;
    const int chunk = blockIdx.x;
    const int t0 = chunk * a.chunk_tiles, t1 = min(t0 + a.chunk_tiles, a.n_tiles);
    for (int col0 = 0; col0 < a.stride; col0 += kPlanThreads) {
        const int ncol = min(a.stride - col0, kPlanThreads);
        const int pad = (ncol + kWave - 1) / kWave * kWave;
        const int parts = kPlanThreads / pad;
        const int part = tid / pad, b = tid - part * pad;
        acc[tid] = 0;
        __syncthreads();
        if (part < parts && b < ncol) {
            const int32_t *h = a.tile_hist + col0 + b;
            int sum = 0;
#pragma unroll 8
            for (int tl = t0 + part; tl < t1; tl += parts) sum += h[(int64_t)tl * a.stride];
            atomicAdd(&acc[b], sum);
        }
        __syncthreads();
        if (tid < ncol) a.chunk_hist[(int64_t)chunk * a.stride + col0 + tid] = acc[tid];
        __syncthreads();
    }
}

// Shared LDS state of the placement kernel.
struct PlaceLds {
    int16_t tile_dev[kTilePairs];              // device of every pair, -1 for an invalid expert id
    int tile_row[kTilePairs];                  // send row of the pairs that are first appearances
    int tile_slot[kTilePairs];                 // expert-major slot of every pair (kept for the fused dispatch)
    uint16_t wave_cnt[kPlanWaves][kMaxBins];   // per wave and key: running count, then prefix over waves
    int base[kMaxBins];                        // per key: pairs in earlier tiles, then the tile's global start
    int total[kMaxBins + 1];
    int invalid;
};

// Stable ranking of the tile's participating pairs by key, in pair order, on top of the global
// order of tiles.  key[r] is the key of pair (wave chunk + r * 64 + lane), or -1 if that pair
// does not take part.  On return pos[r] is the pair's global position: (global exclusive offset
// of its key) + (pairs with that key in earlier tiles) + (earlier pairs with that key in this
// tile).  Block 0 also writes the per-key counts and their exclusive prefix sum.
template <bool SINGLE>
__device__ __forceinline__ void rank_by_key(PlaceLds &s, const PlanArgs &a, int tile, bool writer,
                                            const int (&key)[kRounds], int nb, int hist_off, int32_t *count_out,
                                            int32_t *off_out, int (&pos)[kRounds])
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int nbits = bits_for(nb);
    const uint64_t lt = ((uint64_t)1 << lane) - 1;

    for (int b = lane; b < nb; b += kWave) s.wave_cnt[wave][b] = 0;
    for (int b = tid; b < nb; b += kPlanThreads) {
        s.total[b] = 0;
        s.base[b] = 0;
    }
    __syncthreads();

    // rank inside the wave's chunk; wave_cnt[wave][key] is the running count of the key
    int rank[kRounds];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const bool part = key[r] >= 0;
        const uint64_t m = same_key_lanes(key[r], part, nbits);
        const int before = part ? s.wave_cnt[wave][key[r]] : 0;
        rank[r] = before + __builtin_popcountll(m & lt);
        wave_lds_order();
        if (part && (m & lt) == 0) s.wave_cnt[wave][key[r]] = (uint16_t)(before + __builtin_popcountll(m));
        wave_lds_order();
    }
    __syncthreads();

    // per key: total over all tiles and the part that lies in earlier tiles.  The workgroup splits
    // the tiles into as many interleaved parts as it has groups of nb threads, so that every
    // thread keeps only a few independent loads in flight; partial sums meet in LDS.
    if constexpr (SINGLE) {
        for (int b = tid; b < nb; b += kPlanThreads) {
            int tot = 0;
            for (int w = 0; w < kPlanWaves; ++w) tot += s.wave_cnt[w][b];
            s.total[b] = tot;
        }
    } else {
        const int nb_pad = (nb + kWave - 1) / kWave * kWave;
        const int parts = kPlanThreads / nb_pad;     // >= 1 because nb <= kMaxBins == kPlanThreads
        const int part = tid / nb_pad, b = tid - part * nb_pad;
        if (part < parts && b < nb) {
            const int32_t *h = a.tile_hist + hist_off + b;
            const int me = tile;
            int tot = 0, pre = 0;
            if (a.chunk_tiles == 0) {
#pragma unroll 8
                for (int tl = part; tl < a.n_tiles; tl += parts) {
                    const int v = h[(int64_t)tl * a.stride];
                    tot += v;
                    pre += tl < me ? v : 0;
                }
            } else {
                // whole chunks from their sums, then the tiles of this workgroup's own chunk before it
                const int32_t *ch = a.chunk_hist + hist_off + b;
                const int my_chunk = me / a.chunk_tiles;
#pragma unroll 8
                for (int c = part; c < a.n_chunks; c += parts) {
                    const int v = ch[(int64_t)c * a.stride];
                    tot += v;
                    pre += c < my_chunk ? v : 0;
                }
#pragma unroll 8
                for (int tl = my_chunk * a.chunk_tiles + part; tl < me; tl += parts) pre += h[(int64_t)tl * a.stride];
            }
            atomicAdd(&s.total[b], tot);
            atomicAdd(&s.base[b], pre);
        }
    }
    __syncthreads();
    if (writer && tile == 0)
        for (int b = tid; b < nb; b += kPlanThreads) count_out[b] = s.total[b];

    // exclusive prefix sum over the keys, by wave 0: each lane owns a run of consecutive keys
    if (wave == 0) {
        const int per = (nb + kWave - 1) / kWave;
        const int lo = min(lane * per, nb), hi = min(lo + per, nb);
        int sum = 0;
        for (int b = lo; b < hi; ++b) sum += s.total[b];
        int incl = sum;
        for (int d = 1; d < kWave; d <<= 1) {
            const int up = __shfl_up(incl, d, kWave);
            if (lane >= d) incl += up;
        }
        int run = incl - sum;
        for (int b = lo; b < hi; ++b) {
            const int v = s.total[b];
            s.total[b] = run;
            run += v;
        }
        if (lane == kWave - 1) s.total[nb] = incl;
    }
    __syncthreads();
    if (writer && tile == 0)
        for (int b = tid; b <= nb; b += kPlanThreads) off_out[b] = s.total[b];

    // per key: prefix of the per-wave counts, and the global position where the tile's run starts
    for (int b = tid; b < nb; b += kPlanThreads) {
        int run = 0;
        for (int w = 0; w < kPlanWaves; ++w) {
            const int c = s.wave_cnt[w][b];
            s.wave_cnt[w][b] = (uint16_t)run;
            run += c;
        }
        s.base[b] += s.total[b];
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRounds; ++r)
        pos[r] = key[r] >= 0 ? s.base[key[r]] + s.wave_cnt[wave][key[r]] + rank[r] : -1;
    __syncthreads();
}

// Placement of one tile by one workgroup: pass 2 of the multi-tile planner, or the whole plan when the
// input is a single tile.  A writer stores every descriptor array; a workgroup that is not a writer only
// keeps the tile's slots in LDS (the fused plan + dispatch kernel runs the single-tile plan redundantly in
// every workgroup and lets one of them write it out).
template <bool SINGLE>
__device__ __forceinline__ void place_tile(PlaceLds &s, const PlanArgs &a, int tile, bool writer)
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int tok0 = tile * a.tpt;
    const int ntok = min(a.tpt, a.N - tok0);
    const int npairs = ntok > 0 ? ntok * a.k : 0;
    const int64_t pair0 = (int64_t)tok0 * a.k;

    if (tid == 0) s.invalid = 0;
    __syncthreads();
    int ekey[kRounds], tl[kRounds];   // expert id and tile-local token of the thread's pairs
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = wave * kWaveChunk + r * kWave + lane;
        int key = -1;
        if (p < npairs) {
            const int e = a.A[pair0 + p];
            if ((unsigned)e < (unsigned)a.E) key = e;
            else if constexpr (SINGLE) atomicAdd(&s.invalid, 1);
        }
        tl[r] = div20(p, a.k_magic);
        ekey[r] = key;
        s.tile_dev[p] = (int16_t)(key >= 0 ? div20(key, a.eloc_magic) : -1);
    }
    __syncthreads();

    // level 2 receive side: expert-major slot of every pair
    int slot[kRounds];
    rank_by_key<SINGLE>(s, a, tile, writer, ekey, a.E, 0, a.exp_count, a.exp_off, slot);
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = wave * kWaveChunk + r * kWave + lane;
        s.tile_slot[p] = slot[r];
        if (writer && p < npairs) {
            a.pair_slot[pair0 + p] = slot[r];
            if (slot[r] >= 0) {
                a.slot_pair[slot[r]] = (int32_t)(pair0 + p);
                a.slot_token[slot[r]] = tok0 + tl[r];
            }
        }
    }

    if (!writer) return;   // only the slots are wanted (uniform over the workgroup)

    // level 1: one send row per (token, device), taken at the device's first appearance
    const int dbits = bits_for(a.D);
    int dkey[kRounds], jfirst[kRounds];   // jfirst: the token's first pair on the same device
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = wave * kWaveChunk + r * kWave + lane;
        const int d = s.tile_dev[p];
        uint64_t same;
        jfirst[r] = first_pair_on_device(s.tile_dev, p, lane, tl[r] * a.k, d, dbits, same);
        dkey[r] = jfirst[r] == p ? d : -1;
    }
    int row[kRounds];
    rank_by_key<SINGLE>(s, a, tile, writer, dkey, a.D, a.E, a.send_count, a.send_off, row);
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = wave * kWaveChunk + r * kWave + lane;
        s.tile_row[p] = row[r];
        if (writer && p < npairs) {
            a.pair_first[pair0 + p] = row[r] >= 0 ? 1 : 0;
            if (row[r] >= 0) a.send_src[row[r]] = tok0 + tl[r];
        }
    }
    __syncthreads();

    // level 2 send side: every pair points at the send row of its token on its device
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = wave * kWaveChunk + r * kWave + lane;
        if (!writer || p >= npairs) continue;
        int srow = -1;
        if (ekey[r] >= 0) {
            srow = s.tile_row[jfirst[r]];
            a.slot_send_row[slot[r]] = srow;
        }
        a.pair_send_row[pair0 + p] = srow;
    }

    if (writer && tile == 0 && wave == 0) {
        int bad = 0;
        if constexpr (SINGLE) {
            bad = s.invalid;
        } else {
            // the last column of the counts holds the invalid ids of a tile (or of a chunk of tiles)
            const int32_t *col = (a.chunk_tiles ? a.chunk_hist : a.tile_hist) + a.E + a.D;
            const int rows = a.chunk_tiles ? a.n_chunks : a.n_tiles;
            for (int r = lane; r < rows; r += kWave) bad += col[(int64_t)r * a.stride];
            for (int d = kWave / 2; d > 0; d >>= 1) bad += __shfl_down(bad, d, kWave);
        }
        if (lane == 0) *a.status = bad;
    }
}

template <bool SINGLE>
__global__ __launch_bounds__(kPlanThreads) void plan_place_kernel(PlanArgs a)
{
    __shared__ PlaceLds s;
    place_tile<SINGLE>(s, a, blockIdx.x, true);
}

// ------------------------------------------------------------------------------------------
// Movers.  Both give one workgroup to one token, because HBM rewards long bursts: a row is
// fetched or written whole by neighbouring waves of one compute unit within a short time.
// Measured on MI355X at 14 KiB rows: scattered row reads reach the streaming read rate, scattered
// row writes do not (about 5.2 of 6.9 TB/s), so the movers keep the scattered side of dispatch
// as short as possible (plain cached stores, several chunks per thread in flight).
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ u32x4 load16_stream(const u32x4 *p) { return __builtin_nontemporal_load(p); }

// 16-byte / 8-byte stores that go to memory at system scope instead of lingering in the L2:
// used for the token-ordered output of combine, which is never read again by this kernel.
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

// Dispatch: the row is held in registers between the single read and the k (+ wire) writes.
// Slot lookups depend only on blockIdx, so they are scalar loads.
struct DispatchArgs {
    const u32x4 *x, *x_aux;
    u32x4 *expert_buf, *expert_aux, *send_buf, *send_aux;
    const int32_t *pair_slot, *pair_send_row;
    const uint8_t *pair_first;
    int32_t k;
    int32_t C, Ca;   // 16-byte chunks per row in the main and in the aux plane
    int32_t write_expert, write_wire;
};

template <int CPT>
__global__ __launch_bounds__(256) void dispatch_kernel(DispatchArgs a)
{
    const int t = blockIdx.x;
    const int Ct = a.C + a.Ca;
    const int c0 = blockIdx.y * (blockDim.x * CPT) + threadIdx.x;
    u32x4 v[CPT];
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        const int c = c0 + i * blockDim.x;
        if (c < a.C) v[i] = load16_stream(a.x + (size_t)t * a.C + c);
        else if (c < Ct) v[i] = load16_stream(a.x_aux + (size_t)t * a.Ca + (c - a.C));
    }
    const int32_t *slots = a.pair_slot + (size_t)t * a.k;
    if (a.write_expert) {
        for (int j = 0; j < a.k; ++j) {
            const int slot = slots[j];
            if (slot < 0) continue;
#pragma unroll
            for (int i = 0; i < CPT; ++i) {
                const int c = c0 + i * blockDim.x;
                if (c < a.C) a.expert_buf[(size_t)slot * a.C + c] = v[i];
                else if (c < Ct) a.expert_aux[(size_t)slot * a.Ca + (c - a.C)] = v[i];
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
                if (c < a.C) a.send_buf[(size_t)row * a.C + c] = v[i];
                else if (c < Ct) a.send_aux[(size_t)row * a.Ca + (c - a.C)] = v[i];
            }
        }
    }
}

// Planner and dispatch in one launch for inputs of a single planner tile (decode-sized batches, where
// three dependent launches cost more than the work): one workgroup per token, every workgroup works out the
// whole plan in its own LDS (a few microseconds, all in parallel), workgroup 0 writes the descriptor
// arrays, and each workgroup then moves its token's row to the slots it has just computed.  The row is
// requested before the planning starts, so that its latency hides behind it.
constexpr int kFusedPreload = 4;   // 16-byte chunks per thread held in registers across the planning

__global__ __launch_bounds__(kPlanThreads) void plan_dispatch_kernel(PlanArgs a, DispatchArgs m)
{
    __shared__ PlaceLds s;
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
    place_tile<true>(s, a, 0, blockIdx.x == 0);
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
    // last row first: when combine follows dispatch, the rows written last are the ones still in
    // the memory-side cache
    const int r = gridDim.x - 1 - blockIdx.x;   // token, or send row in the per-send-row mode
    int t = r;
    if constexpr (PER_SEND_ROW) {
        if (r >= *a.n_rows_dev) return;
        t = a.send_src[r];
    }
    const int c0 = blockIdx.y * (blockDim.x * CPT) + threadIdx.x;
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

// ------------------------------------------------------------------------------------------
// Segment-descriptor engine: segments of any size (multiples of 16 bytes) described by
// (offset, size) lists.  The active segment of a stream position is found from the cumulative
// bytes, as in the paper's dense descriptor arrays.
// ------------------------------------------------------------------------------------------
constexpr int kScanThreads = 1024;
constexpr int kSegBlockBytes = 16384;   // stream bytes handled by one workgroup of the copy kernel
constexpr int kSegThreads = 256;
constexpr int kSegUnits = kSegBlockBytes / 16 / kSegThreads;   // 16-byte units per thread

// cum[0] = 0, cum[i + 1] = cum[i] + size of segment i; a descriptor whose offset or size is not a
// multiple of 16 is counted in *status and takes part with size 0.  One workgroup.
__global__ __launch_bounds__(kScanThreads) void segments_scan_kernel(const fusco_segment *desc, int64_t n, uint64_t *cum,
                                                                    int32_t *status)
{
    __shared__ uint64_t part[kScanThreads];
    __shared__ int bad_total;
    const int tid = threadIdx.x;
    const int64_t per = (n + kScanThreads - 1) / kScanThreads;
    const int64_t lo = min((int64_t)tid * per, n), hi = min(lo + per, n);
    if (tid == 0) bad_total = 0;
    __syncthreads();
    uint64_t sum = 0;
    int bad = 0;
    for (int64_t i = lo; i < hi; ++i) {
        const fusco_segment d = desc[i];
        if ((d.offset | d.size) & 15u) ++bad;
        else sum += d.size;
    }
    part[tid] = sum;
    if (bad) atomicAdd(&bad_total, bad);
    __syncthreads();
    for (int d = 1; d < kScanThreads; d <<= 1) {   // inclusive scan of the per-thread sums
        const uint64_t v = tid >= d ? part[tid - d] : 0;
        __syncthreads();
        part[tid] += v;
        __syncthreads();
    }
    uint64_t run = part[tid] - sum;
    for (int64_t i = lo; i < hi; ++i) {
        const fusco_segment d = desc[i];
        cum[i] = run;
        if (!((d.offset | d.size) & 15u)) run += d.size;
    }
    if (tid == kScanThreads - 1) cum[n] = part[tid];
    if (tid == 0) *status = bad_total;
}

__global__ __launch_bounds__(256) void fill_u32_kernel(uint32_t *p, int64_t n, uint32_t v)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

struct SegCopyArgs {
    const char *src;
    char *dst;
    const fusco_segment *src_desc, *dst_desc;   // nullptr: that side is the contiguous stream
    const uint64_t *cum;
    int64_t n;
    uint64_t src_bytes, dst_bytes;
    uint64_t slice_bytes;
    uint32_t *slice_fill;
    int32_t *status;
};

template <bool SLICES>
__global__ __launch_bounds__(kSegThreads) void segments_copy_kernel(SegCopyArgs a)
{
    const uint64_t total = a.cum[a.n];
    const uint64_t base = (uint64_t)blockIdx.x * kSegBlockBytes;
    if (base >= total) return;
    // segment of the workgroup's first byte: last i with cum[i] <= base (uniform, scalar loads)
    int64_t lo = 0, hi = a.n;   // invariant: cum[lo] <= base < cum[hi]
    while (hi - lo > 1) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (a.cum[mid] <= base) lo = mid;
        else hi = mid;
    }
    int64_t i = lo;
    u32x4 v[kSegUnits];
    uint64_t dst_at[kSegUnits];
    bool ok[kSegUnits];
    int skipped = 0;
#pragma unroll
    for (int r = 0; r < kSegUnits; ++r) {
        const uint64_t pos = base + ((uint64_t)r * kSegThreads + threadIdx.x) * 16;
        ok[r] = false;
        if (pos >= total) continue;
        while (a.cum[i + 1] <= pos) ++i;            // i + 1 <= n because pos < cum[n]
        const uint64_t intra = pos - a.cum[i];
        const uint64_t so = a.src_desc ? a.src_desc[i].offset + intra : pos;
        const uint64_t dofs = a.dst_desc ? a.dst_desc[i].offset + intra : pos;
        if (((so | dofs) & 15u) || so + 16 > a.src_bytes || dofs + 16 > a.dst_bytes) {
            ++skipped;
            continue;
        }
        ok[r] = true;
        dst_at[r] = dofs;
        v[r] = *(const u32x4 *)(a.src + so);
    }
#pragma unroll
    for (int r = 0; r < kSegUnits; ++r) {
        if (!ok[r]) continue;
        if constexpr (SLICES) store16_through((u32x4 *)(a.dst + dst_at[r]), v[r]);
        else *(u32x4 *)(a.dst + dst_at[r]) = v[r];
    }
    if (skipped) atomicAdd(a.status, skipped);
    if constexpr (SLICES) {
        // A slice counts bytes only once they are in memory: the stores above go through the L2 at
        // system scope, every thread waits for its own to complete, and only then one thread adds
        // the workgroup's bytes with a system-scope atomic.  (A device-wide release fence would do
        // too, but it writes back the whole L2 of the XCD each time.)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (threadIdx.x == 0) {
            const uint64_t left = total - base;
            __hip_atomic_fetch_add(a.slice_fill + base / a.slice_bytes,
                                   (uint32_t)(left < kSegBlockBytes ? left : kSegBlockBytes), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
}

__global__ __launch_bounds__(256) void probe_copy_kernel(u32x4 *dst, const u32x4 *src, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = load16_stream(src + i);
}

// Measurement aid: row traffic of a chosen shape with no planning and no arithmetic.  Workgroup b reads
// R rows of `src` and writes W rows of `dst`; row i of a stream sits at (i * mul) mod rows, so mul == 1
// walks the buffer in launch order and a multiplier coprime to the row count scatters the rows the way
// a routed shuffle does.  The rows read are XOR-ed so that every load is live.
struct ProbeRowsArgs {
    const u32x4 *src;
    u32x4 *dst;
    uint32_t *sink;
    uint32_t src_rows, dst_rows;
    uint32_t src_mul, dst_mul;
    uint32_t C;          // 16-byte units per row
    uint32_t through;    // 1: write-through stores
};

template <int R, int W>
__global__ __launch_bounds__(256) void probe_rows_kernel(ProbeRowsArgs a)
{
    const uint32_t b = blockIdx.x;
    size_t src_row[R > 0 ? R : 1], dst_row[W > 0 ? W : 1];
#pragma unroll
    for (int i = 0; i < R; ++i)
        src_row[i] = (size_t)(((uint64_t)b * R + i) * a.src_mul % a.src_rows) * a.C;
#pragma unroll
    for (int i = 0; i < W; ++i)
        dst_row[i] = (size_t)(((uint64_t)b * W + i) * a.dst_mul % a.dst_rows) * a.C;
    u32x4 seen = {0u, 0u, 0u, 0u};
    for (uint32_t c = threadIdx.x; c < a.C; c += 256) {
        u32x4 v[R > 0 ? R : 1];
        u32x4 acc = {R == 0 ? b : 0u, R == 0 ? c : 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < R; ++i) v[i] = load16_stream(a.src + src_row[i] + c);
#pragma unroll
        for (int i = 0; i < R; ++i) acc ^= v[i];
#pragma unroll
        for (int i = 0; i < W; ++i) {
            if (a.through) store16_through(a.dst + dst_row[i] + c, acc);
            else a.dst[dst_row[i] + c] = acc;
        }
        seen ^= acc;
    }
    if (W == 0 && (seen.x ^ seen.y ^ seen.z ^ seen.w) == 0x9E3779B9u && a.sink) a.sink[0] = b;
}


bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

// odd multiplier close to frac * n that shares no factor with n: i -> i * mul mod n is a bijection of
// [0, n) that sends neighbours far apart
uint32_t coprime_near(uint32_t n, double frac)
{
    if (n < 3) return 1u;
    uint32_t m = (uint32_t)((double)n * frac) | 1u;
    for (;; m += 2) {
        uint32_t x = n, y = m % n;
        while (y) { const uint32_t r = x % y; x = y; y = r; }
        if (x == 1 && m % n != 0) return m % n;
    }
}

int round_up(int v, int m) { return (v + m - 1) / m * m; }

int launch_status()
{
    return hipGetLastError() == hipSuccess ? FUSCO_OK : FUSCO_ERR_HIP;
}

// Events armed by fusco_probe_time_next_call for the calling thread (null when not armed), and their
// hand-over to the call that consumes them.
thread_local hipEvent_t g_time_start = nullptr, g_time_stop = nullptr;

struct ArmedEvents {
    hipEvent_t start, stop;
    ArmedEvents() : start(g_time_start), stop(g_time_stop)
    {
        g_time_start = nullptr;
        g_time_stop = nullptr;
    }
};

// Kernel launch that can carry a start and a stop event of its own: hipExtLaunchKernelGGL records them
// from the dispatch's own timestamps, without the barrier that a stream event puts between kernels.
template <typename K, typename A>
void launch(K kernel, dim3 grid, dim3 block, hipStream_t s, const A &a, hipEvent_t e0 = nullptr, hipEvent_t e1 = nullptr)
{
    if (e0 || e1) hipExtLaunchKernelGGL(kernel, grid, block, 0, s, e0, e1, 0, a);
    else hipLaunchKernelGGL(kernel, grid, block, 0, s, a);
}

template <bool Y_BF16, bool OUT_BF16>
void launch_combine(const CombineArgs &a, int N, int threads, hipStream_t s, hipEvent_t e0, hipEvent_t e1)
{
    const dim3 grid((unsigned)N, (unsigned)((a.C + threads - 1) / threads)), block((unsigned)threads);
    launch(combine_kernel<Y_BF16, OUT_BF16, 1, 8>, grid, block, s, a, e0, e1);
}

// dst[r] = src[index(r)] for n_rows destination rows of C chunks (see gather_rows_kernel)
template <bool STREAM_LOAD>
void launch_gather(const void *src, void *dst, const int32_t *idx1, const int32_t *idx2, const int32_t *n_rows_dev,
                   int n_rows, int C, hipStream_t s)
{
    if (n_rows <= 0 || C <= 0) return;
    GatherArgs a;
    a.src = (const u32x4 *)src; a.dst = (u32x4 *)dst;
    a.idx1 = idx1; a.idx2 = idx2; a.n_rows_dev = n_rows_dev; a.C = C;
    const int cpt = C >= 512 ? 4 : (C >= 128 ? 2 : 1);
    int threads = round_up((C + cpt - 1) / cpt, kWave);
    if (threads > 256) threads = 256;
    const int segs = (C + threads * cpt - 1) / (threads * cpt);
    const dim3 grid((unsigned)n_rows, (unsigned)segs), block((unsigned)threads);
    switch (cpt) {
    case 1: hipLaunchKernelGGL((gather_rows_kernel<1, STREAM_LOAD>), grid, block, 0, s, a); break;
    case 2: hipLaunchKernelGGL((gather_rows_kernel<2, STREAM_LOAD>), grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL((gather_rows_kernel<4, STREAM_LOAD>), grid, block, 0, s, a); break;
    }
}

void launch_copy(void *dst, const void *src, size_t bytes, hipStream_t s)
{
    const size_t n = bytes / 16;
    if (n == 0) return;
    hipLaunchKernelGGL(probe_copy_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (u32x4 *)dst,
                       (const u32x4 *)src, n);
}

// `empty`: the layout has no tokens, so the tensors hold no rows and may be NULL
int combine_check(const void *d_y, int y_dtype, const float *d_w, const void *d_out, int out_dtype, int32_t H,
                  bool empty)
{
    if (H <= 0 || (!empty && (!d_y || !d_w || !d_out))) return FUSCO_ERR_INVALID_ARG;
    if ((y_dtype != FUSCO_BF16 && y_dtype != FUSCO_F32) || (out_dtype != FUSCO_BF16 && out_dtype != FUSCO_F32))
        return FUSCO_ERR_UNSUPPORTED;
    const size_t y_row = (size_t)H * (y_dtype == FUSCO_BF16 ? 2 : 4);
    if (y_row % 16 != 0 || y_row / 16 > kMaxRowChunks) return FUSCO_ERR_INVALID_ARG;
    if (!aligned16(d_y) || !aligned16(d_out) || ((uintptr_t)d_w & 3u)) return FUSCO_ERR_INVALID_ARG;
    return FUSCO_OK;
}

// out[t] = sum_j w[t, j] * y[pair_slot[t * k + j]] for N tokens; arguments already checked
void combine_launch(const int32_t *pair_slot, int N, int k, const void *d_y, int y_dtype, const float *d_w,
                    void *d_out, int out_dtype, int32_t H, hipStream_t s, hipEvent_t e0 = nullptr,
                    hipEvent_t e1 = nullptr)
{
    CombineArgs a;
    a.y = (const u32x4 *)d_y;
    a.w = d_w;
    a.out = d_out;
    a.pair_slot = pair_slot;
    a.k = k;
    a.pair_send_row = nullptr; a.send_src = nullptr; a.n_rows_dev = nullptr;
    a.C = (int32_t)((size_t)H * (y_dtype == FUSCO_BF16 ? 2 : 4) / 16);
    // one workgroup per token whenever the row fits 1024 threads
    int threads = round_up(a.C, kWave);
    if (threads > 1024) threads = 1024;
    if (y_dtype == FUSCO_BF16 && out_dtype == FUSCO_BF16) launch_combine<true, true>(a, N, threads, s, e0, e1);
    else if (y_dtype == FUSCO_BF16) launch_combine<true, false>(a, N, threads, s, e0, e1);
    else if (out_dtype == FUSCO_BF16) launch_combine<false, true>(a, N, threads, s, e0, e1);
    else launch_combine<false, false>(a, N, threads, s, e0, e1);
}

}   // namespace

extern "C" {

int fusco_version(void) { return FUSCO_VERSION; }

const char *fusco_status_string(int status)
{
    switch (status) {
    case FUSCO_OK: return "ok";
    case FUSCO_ERR_INVALID_ARG: return "invalid argument";
    case FUSCO_ERR_WORKSPACE: return "caller-provided memory too small";
    case FUSCO_ERR_UNSUPPORTED: return "unsupported dtype or flags";
    case FUSCO_ERR_HIP: return "HIP launch failed";
    default: return "unknown status";
    }
}

// Descriptor arrays in the order they are carved; every array starts on a 256-byte boundary.
static size_t layout_carve(fusco_layout *L, int32_t N, int32_t k, int32_t E, int32_t D, char *base)
{
    const size_t P = (size_t)N * k;
    const size_t send_cap = (size_t)N * (size_t)(k < D ? k : D);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *p = base ? base + off : nullptr;
        off += align_up(bytes ? bytes : 1, 256);
        return p;
    };
    int32_t *exp_count = (int32_t *)take((size_t)E * 4);
    int32_t *exp_off = (int32_t *)take((size_t)(E + 1) * 4);
    int32_t *send_count = (int32_t *)take((size_t)D * 4);
    int32_t *send_off = (int32_t *)take((size_t)(D + 1) * 4);
    int32_t *status = (int32_t *)take(4);
    int32_t *pair_slot = (int32_t *)take(P * 4);
    int32_t *slot_pair = (int32_t *)take(P * 4);
    int32_t *slot_token = (int32_t *)take(P * 4);
    int32_t *send_src = (int32_t *)take(send_cap * 4);
    int32_t *pair_send_row = (int32_t *)take(P * 4);
    int32_t *slot_send_row = (int32_t *)take(P * 4);
    uint8_t *pair_first = (uint8_t *)take(P);
    if (L) {
        L->N = N; L->k = k; L->E = E; L->D = D; L->P = (int32_t)P; L->send_cap = (int32_t)send_cap;
        L->exp_count = exp_count; L->exp_off = exp_off; L->send_count = send_count; L->send_off = send_off;
        L->status = status; L->pair_slot = pair_slot; L->slot_pair = slot_pair; L->slot_token = slot_token;
        L->send_src = send_src; L->pair_send_row = pair_send_row; L->slot_send_row = slot_send_row;
        L->pair_first = pair_first;
    }
    return off;
}

size_t fusco_layout_bytes(int32_t N, int32_t k, int32_t E, int32_t D)
{
    if (!sizes_ok(N, k, E, D)) return 0;
    return layout_carve(nullptr, N, k, E, D, nullptr);
}

size_t fusco_scratch_bytes(int32_t N, int32_t k, int32_t E, int32_t D)
{
    if (!sizes_ok(N, k, E, D)) return 0;
    const int tiles = num_tiles(N, k);
    return align_up(((size_t)tiles + (size_t)num_chunks(tiles)) * (size_t)(E + D + 1) * 4, 256);
}

int fusco_layout_bind(fusco_layout *L, int32_t N, int32_t k, int32_t E, int32_t D, void *d_mem, size_t bytes)
{
    if (!L || !d_mem || !sizes_ok(N, k, E, D)) return FUSCO_ERR_INVALID_ARG;
    if (((uintptr_t)d_mem & 255u) != 0) return FUSCO_ERR_INVALID_ARG;
    if (bytes < layout_carve(nullptr, N, k, E, D, nullptr)) return FUSCO_ERR_WORKSPACE;
    layout_carve(L, N, k, E, D, (char *)d_mem);
    return FUSCO_OK;
}

static bool layout_ok(const fusco_layout *L)
{
    if (!L || !sizes_ok(L->N, L->k, L->E, L->D)) return false;
    if ((int64_t)L->P != (int64_t)L->N * L->k) return false;
    return L->exp_count && L->exp_off && L->send_count && L->send_off && L->pair_slot && L->slot_pair &&
           L->slot_token && L->send_src && L->pair_send_row && L->slot_send_row && L->pair_first && L->status;
}

static PlanArgs plan_args(const fusco_layout *L, const int32_t *d_topk_idx, void *d_scratch)
{
    PlanArgs a;
    a.A = d_topk_idx;
    a.N = L->N; a.k = L->k; a.E = L->E; a.D = L->D; a.Eloc = L->E / L->D;
    a.k_magic = ((1u << 20) + a.k - 1) / a.k;
    a.eloc_magic = ((1u << 20) + a.Eloc - 1) / a.Eloc;
    a.tpt = tokens_per_tile(L->k);
    a.n_tiles = num_tiles(L->N, L->k);
    a.stride = L->E + L->D + 1;
    a.tile_hist = (int32_t *)d_scratch;   // unused (may be NULL) when the input is a single tile
    a.chunk_tiles = chunk_tiles_for(a.n_tiles);
    a.n_chunks = num_chunks(a.n_tiles);
    a.chunk_hist = a.tile_hist + (size_t)a.n_tiles * (size_t)a.stride;
    a.exp_count = L->exp_count; a.exp_off = L->exp_off; a.send_count = L->send_count; a.send_off = L->send_off;
    a.pair_slot = L->pair_slot; a.slot_pair = L->slot_pair; a.slot_token = L->slot_token; a.send_src = L->send_src;
    a.pair_send_row = L->pair_send_row; a.slot_send_row = L->slot_send_row; a.pair_first = L->pair_first;
    a.status = L->status;
    return a;
}

int fusco_plan(fusco_layout *L, const int32_t *d_topk_idx, void *d_scratch, size_t scratch_bytes, void *stream)
{
    if (!layout_ok(L) || (!d_topk_idx && L->N > 0) || !d_scratch) return FUSCO_ERR_INVALID_ARG;
    if (scratch_bytes < fusco_scratch_bytes(L->N, L->k, L->E, L->D)) return FUSCO_ERR_WORKSPACE;
    const PlanArgs a = plan_args(L, d_topk_idx, d_scratch);
    hipStream_t s = (hipStream_t)stream;
    const ArmedEvents ev;
    if (a.n_tiles == 1) {
        launch(plan_place_kernel<true>, dim3(1), dim3(kPlanThreads), s, a, ev.start, ev.stop);
    } else {
        launch(plan_count_kernel, dim3(a.n_tiles), dim3(kPlanThreads), s, a, ev.start, nullptr);
        if (a.n_chunks > 0) launch(plan_chunk_kernel, dim3(a.n_chunks), dim3(kPlanThreads), s, a);
        launch(plan_place_kernel<false>, dim3(a.n_tiles), dim3(kPlanThreads), s, a, nullptr, ev.stop);
    }
    return launch_status();
}

int fusco_plan_dispatch(fusco_layout *L, const int32_t *d_topk_idx, const void *d_x, size_t row_bytes,
                        const void *d_x_aux, size_t aux_row_bytes, void *d_expert_buf, void *d_expert_aux,
                        void *stream)
{
    if (!layout_ok(L) || (!d_topk_idx && L->N > 0)) return FUSCO_ERR_INVALID_ARG;
    if (row_bytes == 0 || row_bytes % 16 != 0 || aux_row_bytes % 16 != 0) return FUSCO_ERR_INVALID_ARG;
    if ((row_bytes + aux_row_bytes) / 16 > kMaxRowChunks) return FUSCO_ERR_INVALID_ARG;
    if (num_tiles(L->N, L->k) != 1) return FUSCO_ERR_UNSUPPORTED;
    if (L->N > 0) {
        if (!d_x || !d_expert_buf || (aux_row_bytes && (!d_x_aux || !d_expert_aux))) return FUSCO_ERR_INVALID_ARG;
        if (!aligned16(d_x) || !aligned16(d_x_aux) || !aligned16(d_expert_buf) || !aligned16(d_expert_aux))
            return FUSCO_ERR_INVALID_ARG;
    }
    const PlanArgs a = plan_args(L, d_topk_idx, nullptr);
    DispatchArgs m;
    m.x = (const u32x4 *)d_x; m.x_aux = (const u32x4 *)d_x_aux;
    m.expert_buf = (u32x4 *)d_expert_buf; m.expert_aux = (u32x4 *)d_expert_aux;
    m.send_buf = nullptr; m.send_aux = nullptr;
    m.pair_slot = L->pair_slot; m.pair_send_row = L->pair_send_row; m.pair_first = L->pair_first;
    m.k = L->k;
    m.C = (int32_t)(row_bytes / 16); m.Ca = (int32_t)(aux_row_bytes / 16);
    m.write_expert = 1; m.write_wire = 0;
    const ArmedEvents ev;
    const dim3 grid((unsigned)(L->N > 0 ? L->N : 1)), block(kPlanThreads);
    if (ev.start || ev.stop)
        hipExtLaunchKernelGGL(plan_dispatch_kernel, grid, block, 0, (hipStream_t)stream, ev.start, ev.stop, 0, a, m);
    else
        hipLaunchKernelGGL(plan_dispatch_kernel, grid, block, 0, (hipStream_t)stream, a, m);
    return launch_status();
}

int fusco_dispatch(const fusco_layout *L, const void *d_x, size_t row_bytes, const void *d_x_aux,
                   size_t aux_row_bytes, void *d_expert_buf, void *d_expert_aux, void *d_send_buf,
                   void *d_send_aux, uint32_t flags, void *stream)
{
    if (!layout_ok(L)) return FUSCO_ERR_INVALID_ARG;
    if (flags == 0) flags = FUSCO_DISPATCH_EXPERT;
    if (flags & ~(FUSCO_DISPATCH_EXPERT | FUSCO_DISPATCH_WIRE | FUSCO_DISPATCH_TWO_HOP)) return FUSCO_ERR_UNSUPPORTED;
    const bool two_hop = flags & FUSCO_DISPATCH_TWO_HOP;
    if (two_hop) flags |= FUSCO_DISPATCH_EXPERT | FUSCO_DISPATCH_WIRE;   // both tensors are produced
    const bool expert = flags & FUSCO_DISPATCH_EXPERT, wire = flags & FUSCO_DISPATCH_WIRE;
    if (row_bytes == 0 || row_bytes % 16 != 0 || aux_row_bytes % 16 != 0) return FUSCO_ERR_INVALID_ARG;
    if ((row_bytes + aux_row_bytes) / 16 > kMaxRowChunks) return FUSCO_ERR_INVALID_ARG;
    if (L->N == 0) return FUSCO_OK;   // nothing to move: the (empty) tensors may be NULL
    if (!d_x || (aux_row_bytes && !d_x_aux)) return FUSCO_ERR_INVALID_ARG;
    if (expert && (!d_expert_buf || (aux_row_bytes && !d_expert_aux))) return FUSCO_ERR_INVALID_ARG;
    if (wire && (!d_send_buf || (aux_row_bytes && !d_send_aux))) return FUSCO_ERR_INVALID_ARG;
    if (!aligned16(d_x) || !aligned16(d_x_aux) || !aligned16(d_expert_buf) || !aligned16(d_expert_aux) ||
        !aligned16(d_send_buf) || !aligned16(d_send_aux))
        return FUSCO_ERR_INVALID_ARG;

    DispatchArgs a;
    a.x = (const u32x4 *)d_x;
    a.x_aux = (const u32x4 *)d_x_aux;
    a.expert_buf = (u32x4 *)d_expert_buf; a.expert_aux = (u32x4 *)d_expert_aux;
    a.send_buf = (u32x4 *)d_send_buf; a.send_aux = (u32x4 *)d_send_aux;
    a.pair_slot = L->pair_slot; a.pair_send_row = L->pair_send_row; a.pair_first = L->pair_first;
    a.k = L->k;
    a.C = (int32_t)(row_bytes / 16);
    a.Ca = (int32_t)(aux_row_bytes / 16);
    a.write_expert = expert && !two_hop; a.write_wire = wire;
    const int Ct = a.C + a.Ca;

    int cpt = Ct >= 512 ? 4 : (Ct >= 128 ? 2 : 1);
    int threads = round_up((Ct + cpt - 1) / cpt, kWave);
    if (threads > 256) threads = 256;
    const int segs = (Ct + threads * cpt - 1) / (threads * cpt);
    const dim3 grid((unsigned)L->N, (unsigned)segs), block((unsigned)threads);
    hipStream_t s = (hipStream_t)stream;
    ArmedEvents ev;
    if (two_hop) ev.start = ev.stop = nullptr;   // several kernels: armed events are dropped
    switch (cpt) {
    case 1: launch(dispatch_kernel<1>, grid, block, s, a, ev.start, ev.stop); break;
    case 2: launch(dispatch_kernel<2>, grid, block, s, a, ev.start, ev.stop); break;
    default: launch(dispatch_kernel<4>, grid, block, s, a, ev.start, ev.stop); break;
    }
    if (two_hop) {
        // second hop: every row of the expert tensor is pulled from its token's row in the receive
        // tensor of the expert's device (level-2 send descriptor), over the exp_off[E] assigned rows
        launch_gather<false>(d_send_buf, d_expert_buf, L->slot_send_row, nullptr, L->exp_off + L->E, L->P, a.C, s);
        if (a.Ca)
            launch_gather<false>(d_send_aux, d_expert_aux, L->slot_send_row, nullptr, L->exp_off + L->E, L->P, a.Ca, s);
    }
    return launch_status();
}

int fusco_combine(const fusco_layout *L, const void *d_y, int y_dtype, const float *d_w, void *d_out,
                  int out_dtype, int32_t H, uint32_t flags, void *stream)
{
    if (!layout_ok(L)) return FUSCO_ERR_INVALID_ARG;
    if (flags != 0) return FUSCO_ERR_UNSUPPORTED;
    const int rc = combine_check(d_y, y_dtype, d_w, d_out, out_dtype, H, L->N == 0);
    if (rc != FUSCO_OK || L->N == 0) return rc;
    const ArmedEvents ev;
    combine_launch(L->pair_slot, L->N, L->k, d_y, y_dtype, d_w, d_out, out_dtype, H, (hipStream_t)stream, ev.start,
                   ev.stop);
    return launch_status();
}

int fusco_combine_two_hop(const fusco_layout *L, const void *d_y, int y_dtype, const float *d_w, float *d_partial,
                          void *d_out, int out_dtype, int32_t H, void *stream)
{
    if (!layout_ok(L) || (!d_partial && L->N > 0) || !aligned16(d_partial)) return FUSCO_ERR_INVALID_ARG;
    const int rc = combine_check(d_y, y_dtype, d_w, d_out, out_dtype, H, L->N == 0);
    if (rc != FUSCO_OK || L->N == 0) return rc;
    hipStream_t s = (hipStream_t)stream;
    if (L->k <= 8) {
        TwoHopArgs f;
        f.y = (const u32x4 *)d_y; f.w = d_w; f.partial = d_partial; f.out = d_out;
        f.pair_slot = L->pair_slot; f.pair_send_row = L->pair_send_row; f.pair_first = L->pair_first;
        f.k = L->k;
        f.C = (int32_t)((size_t)H * (y_dtype == FUSCO_BF16 ? 2 : 4) / 16);
        int th = round_up(f.C, kWave);
        if (th > 1024) th = 1024;
        const dim3 fgrid((unsigned)L->N, (unsigned)((f.C + th - 1) / th));
        if (y_dtype == FUSCO_BF16 && out_dtype == FUSCO_BF16)
            hipLaunchKernelGGL((combine_two_hop_kernel<true, true>), fgrid, dim3(th), 0, s, f);
        else if (y_dtype == FUSCO_BF16) hipLaunchKernelGGL((combine_two_hop_kernel<true, false>), fgrid, dim3(th), 0, s, f);
        else if (out_dtype == FUSCO_BF16) hipLaunchKernelGGL((combine_two_hop_kernel<false, true>), fgrid, dim3(th), 0, s, f);
        else hipLaunchKernelGGL((combine_two_hop_kernel<false, false>), fgrid, dim3(th), 0, s, f);
        return launch_status();
    }
    // general k: level 2 reversed (fp32 partial row per send row), then level 1 reversed
    CombineArgs a;
    a.y = (const u32x4 *)d_y;
    a.w = d_w;
    a.out = d_partial;
    a.pair_slot = L->pair_slot;
    a.k = L->k;
    a.C = (int32_t)((size_t)H * (y_dtype == FUSCO_BF16 ? 2 : 4) / 16);
    a.pair_send_row = L->pair_send_row; a.send_src = L->send_src; a.n_rows_dev = L->send_off + L->D;
    int threads = round_up(a.C, kWave);
    if (threads > 1024) threads = 1024;
    const dim3 grid((unsigned)L->send_cap, (unsigned)((a.C + threads - 1) / threads));
    if (y_dtype == FUSCO_BF16) hipLaunchKernelGGL((combine_kernel<true, false, 1, 8, true>), grid, dim3(threads), 0, s, a);
    else hipLaunchKernelGGL((combine_kernel<false, false, 1, 8, true>), grid, dim3(threads), 0, s, a);
    // level 1 reversed: sum of the token's partial rows
    SumPartialsArgs b;
    b.partial = (const u32x4 *)d_partial;
    b.out = d_out;
    b.pair_send_row = L->pair_send_row; b.pair_first = L->pair_first;
    b.k = L->k;
    b.C = H / 4;
    int th2 = round_up(b.C, kWave);
    if (th2 > 1024) th2 = 1024;
    const dim3 grid2((unsigned)L->N, (unsigned)((b.C + th2 - 1) / th2));
    if (out_dtype == FUSCO_BF16) hipLaunchKernelGGL(sum_partials_kernel<true>, grid2, dim3(th2), 0, s, b);
    else hipLaunchKernelGGL(sum_partials_kernel<false>, grid2, dim3(th2), 0, s, b);
    return launch_status();
}

int fusco_disaggregated_plan(fusco_layout *Lr, const fusco_layout *L, const int32_t *d_topk_idx, int32_t *d_topk_dev,
                             void *d_scratch, size_t scratch_bytes, void *stream)
{
    if (!layout_ok(L) || !layout_ok(Lr) || (!d_topk_idx && L->N > 0) || (!d_topk_dev && L->N > 0))
        return FUSCO_ERR_INVALID_ARG;
    if (Lr->N != L->N || Lr->k != L->k || Lr->E != L->D || Lr->D != L->D) return FUSCO_ERR_INVALID_ARG;
    if (scratch_bytes < fusco_scratch_bytes(Lr->N, Lr->k, Lr->E, Lr->D)) return FUSCO_ERR_WORKSPACE;
    if (L->P > 0)
        hipLaunchKernelGGL(expert_to_device_kernel, dim3((unsigned)((L->P + 255) / 256)), dim3(256), 0,
                           (hipStream_t)stream, d_topk_dev, d_topk_idx, (int64_t)L->P, L->E, L->E / L->D);
    return fusco_plan(Lr, d_topk_dev, d_scratch, scratch_bytes, stream);
}

static bool rank_layout_matches(const fusco_layout *L, const fusco_layout *Lr)
{
    return layout_ok(L) && layout_ok(Lr) && Lr->N == L->N && Lr->k == L->k && Lr->E == L->D && Lr->D == L->D;
}

int fusco_disaggregated_dispatch(const fusco_layout *L, const fusco_layout *Lr, const void *d_x, size_t row_bytes,
                                 void *d_stage_a, void *d_stage_b, void *d_expert_buf, void *stream)
{
    if (!rank_layout_matches(L, Lr)) return FUSCO_ERR_INVALID_ARG;
    if (row_bytes == 0 || row_bytes % 16 != 0 || row_bytes / 16 > kMaxRowChunks) return FUSCO_ERR_INVALID_ARG;
    if (L->N == 0) return FUSCO_OK;
    if (!d_x || !d_stage_a || !d_stage_b || !d_expert_buf) return FUSCO_ERR_INVALID_ARG;
    if (!aligned16(d_x) || !aligned16(d_stage_a) || !aligned16(d_stage_b) || !aligned16(d_expert_buf))
        return FUSCO_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const int C = (int)(row_bytes / 16);
    // 1) rearrange by destination device: one row per (token, expert) pair, device-major, token order
    launch_gather<false>(d_x, d_stage_a, Lr->slot_token, nullptr, Lr->exp_off + Lr->E, L->P, C, s);
    // 2) the exchange between the virtual devices: a contiguous copy of the packed buffer
    launch_copy(d_stage_b, d_stage_a, (size_t)L->P * row_bytes, s);
    // 3) rearrange the received rows by expert
    launch_gather<true>(d_stage_b, d_expert_buf, L->slot_pair, Lr->pair_slot, L->exp_off + L->E, L->P, C, s);
    return launch_status();
}

int fusco_disaggregated_combine(const fusco_layout *L, const fusco_layout *Lr, const void *d_y, int y_dtype,
                                const float *d_w, void *d_stage_a, void *d_stage_b, void *d_out, int out_dtype,
                                int32_t H, void *stream)
{
    if (!rank_layout_matches(L, Lr)) return FUSCO_ERR_INVALID_ARG;
    const int rc = combine_check(d_y, y_dtype, d_w, d_out, out_dtype, H, L->N == 0);
    if (rc != FUSCO_OK || L->N == 0) return rc;
    if (!d_stage_a || !d_stage_b || !aligned16(d_stage_a) || !aligned16(d_stage_b)) return FUSCO_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const size_t row_bytes = (size_t)H * (y_dtype == FUSCO_BF16 ? 2 : 4);
    // 3') expert order -> rank order, 2') exchange copy, 1') un-permute with the weighted sum
    launch_gather<true>(d_y, d_stage_b, Lr->slot_pair, L->pair_slot, Lr->exp_off + Lr->E, L->P, (int)(row_bytes / 16), s);
    launch_copy(d_stage_a, d_stage_b, (size_t)L->P * row_bytes, s);
    combine_launch(Lr->pair_slot, L->N, L->k, d_stage_a, y_dtype, d_w, d_out, out_dtype, H, s);
    return launch_status();
}

int fusco_balance_groups(const int64_t *load, int32_t nodes, int32_t gpus, int32_t *group_gpu)
{
    if (!load || !group_gpu || nodes < 1 || gpus < 1 || (int64_t)nodes * gpus > (1 << 24)) return FUSCO_ERR_INVALID_ARG;
    int32_t *perm = (int32_t *)malloc((size_t)gpus * sizeof(int32_t));
    if (!perm) return FUSCO_ERR_WORKSPACE;
    for (int32_t n = 0; n < nodes; ++n) {
        const int64_t *l = load + (size_t)n * gpus;
        // P_n: local GPUs by descending load (insertion sort, stable: equal loads keep index order)
        for (int32_t g = 0; g < gpus; ++g) {
            int32_t pos = g;
            while (pos > 0 && l[perm[pos - 1]] < l[g]) {
                perm[pos] = perm[pos - 1];
                --pos;
            }
            perm[pos] = g;
        }
        // S_n: P_n rotated by the node index; group i takes position i of S_n
        for (int32_t i = 0; i < gpus; ++i) group_gpu[(size_t)i * nodes + n] = perm[(i + n) % gpus];
    }
    free(perm);
    return FUSCO_OK;
}

int fusco_segments_scan(const fusco_segment *d_desc, int64_t n, uint64_t *d_cum, int32_t *d_status, void *stream)
{
    if (n < 0 || n > ((int64_t)1 << 26) || !d_cum || !d_status || (n > 0 && !d_desc)) return FUSCO_ERR_INVALID_ARG;
    if (((uintptr_t)d_desc | (uintptr_t)d_cum) & 7u) return FUSCO_ERR_INVALID_ARG;
    hipLaunchKernelGGL(segments_scan_kernel, dim3(1), dim3(kScanThreads), 0, (hipStream_t)stream, d_desc, n, d_cum, d_status);
    return launch_status();
}

int fusco_segments_copy(const void *d_src, uint64_t src_bytes, const fusco_segment *d_src_desc, void *d_dst,
                        uint64_t dst_bytes, const fusco_segment *d_dst_desc, const uint64_t *d_cum, int64_t n,
                        uint64_t stream_capacity, uint64_t slice_bytes, uint32_t *d_slice_fill, int32_t *d_status,
                        void *stream)
{
    if (!d_src || !d_dst || !d_cum || !d_status || n < 0 || n > ((int64_t)1 << 26)) return FUSCO_ERR_INVALID_ARG;
    if (!aligned16(d_src) || !aligned16(d_dst)) return FUSCO_ERR_INVALID_ARG;
    if (d_slice_fill && (slice_bytes == 0 || slice_bytes % kSegBlockBytes != 0 || slice_bytes > ((uint64_t)1 << 31)))
        return FUSCO_ERR_INVALID_ARG;
    const uint64_t blocks = (stream_capacity + kSegBlockBytes - 1) / kSegBlockBytes;
    if (blocks > 0x7FFFFFFFu) return FUSCO_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    if (d_slice_fill) {
        const int64_t slices = (int64_t)((stream_capacity + slice_bytes - 1) / slice_bytes);
        if (slices > 0)
            hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((slices + 255) / 256)), dim3(256), 0, s, d_slice_fill,
                               slices, 0u);
    }
    if (n == 0 || blocks == 0) return launch_status();
    SegCopyArgs a;
    a.src = (const char *)d_src; a.dst = (char *)d_dst;
    a.src_desc = d_src_desc; a.dst_desc = d_dst_desc;
    a.cum = d_cum; a.n = n;
    a.src_bytes = src_bytes; a.dst_bytes = dst_bytes;
    a.slice_bytes = slice_bytes; a.slice_fill = d_slice_fill; a.status = d_status;
    if (d_slice_fill) hipLaunchKernelGGL(segments_copy_kernel<true>, dim3((unsigned)blocks), dim3(kSegThreads), 0, s, a);
    else hipLaunchKernelGGL(segments_copy_kernel<false>, dim3((unsigned)blocks), dim3(kSegThreads), 0, s, a);
    return launch_status();
}

int fusco_probe_copy(void *d_dst, const void *d_src, size_t bytes, void *stream)
{
    if (!d_dst || !d_src || bytes % 16 != 0 || !aligned16(d_dst) || !aligned16(d_src)) return FUSCO_ERR_INVALID_ARG;
    if (bytes == 0) return FUSCO_OK;
    const size_t n = bytes / 16;
    const size_t blocks = (n + 255) / 256;
    if (blocks > 0x7FFFFFFFu) return FUSCO_ERR_INVALID_ARG;
    hipLaunchKernelGGL(probe_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       (u32x4 *)d_dst, (const u32x4 *)d_src, n);
    return launch_status();
}

int fusco_probe_rows(const void *d_src, uint32_t src_rows, void *d_dst, uint32_t dst_rows, size_t row_bytes,
                     int reads_per_group, int writes_per_group, int scatter, int write_through,
                     uint32_t *d_sink, void *stream)
{
    const int R = reads_per_group, W = writes_per_group;
    const bool shape_ok = (R == 0 && W == 1) || (R == 1 && W == 0) || (R == 1 && W == 1) || (R == 1 && W == 8) ||
                          (R == 8 && W == 1);
    if (!shape_ok || row_bytes == 0 || row_bytes % 16 != 0 || row_bytes / 16 > 0xFFFFFFFFu) return FUSCO_ERR_INVALID_ARG;
    if ((R > 0 && (!d_src || !aligned16(d_src) || src_rows == 0)) || (W > 0 && (!d_dst || !aligned16(d_dst) || dst_rows == 0)))
        return FUSCO_ERR_INVALID_ARG;
    if (W == 0 && !d_sink) return FUSCO_ERR_INVALID_ARG;
    // every workgroup moves whole rows: the stream that fixes the grid must divide evenly
    const uint32_t groups = W > 0 ? dst_rows / (uint32_t)W : src_rows / (uint32_t)R;
    if (W > 0 && dst_rows % (uint32_t)W != 0) return FUSCO_ERR_INVALID_ARG;
    if (R > 0 && (uint64_t)groups * (uint64_t)R > src_rows) return FUSCO_ERR_INVALID_ARG;
    if (groups == 0) return FUSCO_OK;
    ProbeRowsArgs a;
    a.src = (const u32x4 *)d_src; a.dst = (u32x4 *)d_dst; a.sink = d_sink;
    a.src_rows = src_rows ? src_rows : 1; a.dst_rows = dst_rows ? dst_rows : 1;
    a.src_mul = scatter ? coprime_near(a.src_rows, 0.3819660112501051) : 1u;
    a.dst_mul = scatter ? coprime_near(a.dst_rows, 0.6180339887498949) : 1u;
    a.C = (uint32_t)(row_bytes / 16); a.through = write_through ? 1u : 0u;
    const dim3 grid(groups), block(256);
    hipStream_t s = (hipStream_t)stream;
    if (R == 0) hipLaunchKernelGGL((probe_rows_kernel<0, 1>), grid, block, 0, s, a);
    else if (W == 0) hipLaunchKernelGGL((probe_rows_kernel<1, 0>), grid, block, 0, s, a);
    else if (R == 1 && W == 1) hipLaunchKernelGGL((probe_rows_kernel<1, 1>), grid, block, 0, s, a);
    else if (R == 1) hipLaunchKernelGGL((probe_rows_kernel<1, 8>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((probe_rows_kernel<8, 1>), grid, block, 0, s, a);
    return launch_status();
}

int fusco_probe_time_next_call(void *start_event, void *stop_event)
{
    if (!start_event || !stop_event) return FUSCO_ERR_INVALID_ARG;
    g_time_start = (hipEvent_t)start_event;
    g_time_stop = (hipEvent_t)stop_event;
    return FUSCO_OK;
}

}   // extern "C"
