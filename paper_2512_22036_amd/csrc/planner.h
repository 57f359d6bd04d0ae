// Planner kernels: token-expert matrix -> two-level layout descriptor (paper section 3.3).
#ifndef FUSCO_CSRC_PLANNER_H
#define FUSCO_CSRC_PLANNER_H

#include "common.h"

namespace {

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
    int32_t *tile_slots;   // [n_tiles][tpt * k]: the slots of a tile's pairs in ascending order, then -1
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
template <int R>
__global__ __launch_bounds__(kPlanThreads) void plan_count_kernel(PlanArgs a)
{
    __shared__ int16_t tile_dev[R * kRoundPairs];
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
    int ekey[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
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
    for (int r = 0; r < R; ++r) {
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
template <int R>
struct PlaceLds {
    int16_t tile_dev[R * kRoundPairs];              // device of every pair, -1 for an invalid expert id
    int tile_row[R * kRoundPairs];                  // send row of the pairs that are first appearances
    int tile_slot[R * kRoundPairs];                 // expert-major slot of every pair (kept for the fused dispatch)
    uint16_t wave_cnt[kPlanWaves][kMaxBins];   // per wave and key: running count, then prefix over waves
    int base[kMaxBins];                        // per key: pairs in earlier tiles, then the tile's global start
    int total[kMaxBins + 1];
    int invalid;
    int tile_pairs;                            // pairs of the tile with a valid expert id
};

// Counts of the other tiles, as the placement kernel needs them: thread (part, b) of the workgroup adds up,
// for key b, the counts of tiles part, part + parts, ... (parts = groups of nb threads that fit the workgroup).
// The first kCross of these loads depend on nothing the workgroup computes; place_tile issues
// them right after its loads of the routing and uses the values only after the ranking inside the tile, so
// that one memory latency is paid instead of three in a row (the counts were written by other XCDs in the
// previous kernel and come from memory).  Not used with a chunk level.
constexpr int kCross = 16;   // 48 tiles of 256 experts + 8 devices are covered without a loop

template <int PF>
__device__ __forceinline__ void cross_prefetch(const PlanArgs &a, int nb, int hist_off, int (&v)[PF])
{
    const int tid = threadIdx.x;
    const int nb_pad = (nb + kWave - 1) / kWave * kWave;
    const int parts = kPlanThreads / nb_pad;
    const int part = tid / nb_pad, b = tid - part * nb_pad;
    const bool active = a.chunk_tiles == 0 && part < parts && b < nb;
    const int32_t *h = a.tile_hist + hist_off + b;
#pragma unroll
    for (int i = 0; i < PF; ++i) {
        const int tl = part + i * parts;
        v[i] = active && tl < a.n_tiles ? h[(int64_t)tl * a.stride] : 0;
    }
}

// Exclusive prefix sum of v[0 .. nb) in place, by the calling wave (all 64 lanes): each lane owns a run of
// consecutive entries; *total receives the sum.
__device__ __forceinline__ void wave_exclusive_scan(int *v, int nb, int *total)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int per = (nb + kWave - 1) / kWave;
    const int lo = min(lane * per, nb), hi = min(lo + per, nb);
    int sum = 0;
    for (int b = lo; b < hi; ++b) sum += v[b];
    int incl = sum;
    for (int d = 1; d < kWave; d <<= 1) {
        const int up = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += up;
    }
    int run = incl - sum;
    for (int b = lo; b < hi; ++b) {
        const int x = v[b];
        v[b] = run;
        run += x;
    }
    if (lane == kWave - 1) *total = incl;
}

// Clears the counters of rank_bins for nb bins.  The caller puts a barrier between this and rank_bins.
template <int R>
__device__ __forceinline__ void rank_clear(PlaceLds<R> &s, int nb)
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    for (int b = lane; b < nb; b += kWave) s.wave_cnt[wave][b] = 0;
    for (int b = tid; b < nb; b += kPlanThreads) {
        s.total[b] = 0;
        s.base[b] = 0;
    }
}

// Stable ranking of the tile's pairs by key, in pair order, on top of the global order of tiles.
// The bins are nE expert bins followed by nD device bins (either may be 0): expert keys are ranked into
// slots of the expert-activation tensor, device keys (first appearances only) into send rows, in one
// pass over a common set of counters.  key[i] is a bin, or -1 for an entry that does not take part; the
// thread's NK entries are ranked in the order i = 0 .. NK-1, each index being one round of 64 consecutive
// pairs of the wave.  On return pos[i] is the entry's global position inside its own family: (exclusive
// offset of the key among the experts, or among the devices) + (entries with that key in earlier tiles) +
// (earlier entries with that key in this tile).  tile_pos[i] is, for expert keys, the position among the
// tile's own pairs in (expert, pair) order; s.tile_pairs receives their number.  Block 0 also writes the
// per-key counts and their exclusive prefix sums.  hist_off: column of bin 0 in the per-tile counts.
// pre_v: the first PF per-tile counts of this thread's key and part (cross_prefetch).
template <bool SINGLE, int R, int NK, int PF>
__device__ __forceinline__ void rank_bins(PlaceLds<R> &s, const PlanArgs &a, int tile, bool writer, const int (&key)[NK],
                                          int nE, int nD, int hist_off, const int (&pre_v)[PF], int (&pos)[NK],
                                          int (&tile_pos)[NK])
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int nb = nE + nD;
    // entries of one index i are all expert keys (i < expert_rounds) or all device keys, so lanes with the
    // same key are found by comparing only as many bits as that family has
    const int expert_rounds = nE == 0 ? 0 : (nD == 0 ? NK : NK / 2);
    const int ebits = bits_for(nE), dbits = bits_for(nD);
    const uint64_t lt = ((uint64_t)1 << lane) - 1;
    int *tile_cnt = s.tile_row;   // the tile's own count per expert, then their prefix: tile_row is written later

    // rank inside the wave's chunk; wave_cnt[wave][key] is the running count of the key (zero on entry:
    // rank_clear, and a barrier, come before this call)
    int rank[NK];
#pragma unroll
    for (int i = 0; i < NK; ++i) {
        const bool part = key[i] >= 0;
        const uint64_t m = i < expert_rounds ? same_key_lanes(key[i], part, ebits) : same_key_lanes(key[i] - nE, part, dbits);
        const int before = part ? s.wave_cnt[wave][key[i]] : 0;
        rank[i] = before + __builtin_popcountll(m & lt);
        wave_lds_order();
        if (part && (m & lt) == 0) s.wave_cnt[wave][key[i]] = (uint16_t)(before + __builtin_popcountll(m));
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
                // the first PF tiles of this part were requested at the start of the kernel
#pragma unroll
                for (int i = 0; i < PF; ++i) {
                    tot += pre_v[i];
                    pre += part + i * parts < me ? pre_v[i] : 0;
                }
#pragma unroll 8
                for (int tl = part + PF * parts; tl < a.n_tiles; tl += parts) {
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
        for (int b = tid; b < nb; b += kPlanThreads) {
            if (b < nE) a.exp_count[b] = s.total[b];
            else a.send_count[b - nE] = s.total[b];
        }

    // exclusive prefix sum over all bins, by wave 0; the devices' offsets start after the experts' total
    if (wave == 0) wave_exclusive_scan(s.total, nb, &s.total[nb]);
    __syncthreads();
    const int experts_total = s.total[nE];   // 0 when there are no expert bins
    if (writer && tile == 0)
        for (int b = tid; b <= nb; b += kPlanThreads) {
            if (nE > 0 && b <= nE) a.exp_off[b] = s.total[b];
            if (nD > 0 && b >= nE) a.send_off[b - nE] = s.total[b] - experts_total;
        }

    // per key: prefix of the per-wave counts, the global position where the tile's run starts, and the
    // tile's own count per expert
    for (int b = tid; b < nb; b += kPlanThreads) {
        int run = 0;
        for (int w = 0; w < kPlanWaves; ++w) {
            const int c = s.wave_cnt[w][b];
            s.wave_cnt[w][b] = (uint16_t)run;
            run += c;
        }
        s.base[b] += s.total[b] - (b >= nE ? experts_total : 0);
        if (b < nE) tile_cnt[b] = run;
    }
    __syncthreads();
    // the tile's own exclusive prefix over the experts gives the order of its pairs by (expert, pair)
    if (wave == 0 && nE > 0) wave_exclusive_scan(tile_cnt, nE, &s.tile_pairs);
#pragma unroll
    for (int i = 0; i < NK; ++i)
        pos[i] = key[i] >= 0 ? s.base[key[i]] + s.wave_cnt[wave][key[i]] + rank[i] : -1;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NK; ++i)
        tile_pos[i] = key[i] >= 0 && key[i] < nE ? tile_cnt[key[i]] + s.wave_cnt[wave][key[i]] + rank[i] : -1;
    __syncthreads();
}

// Placement of one tile by one workgroup: pass 2 of the multi-tile planner, or the whole plan when the
// input is a single tile.  A writer stores every descriptor array; a workgroup that is not a writer only
// keeps the tile's slots in LDS (the fused plan + dispatch kernel runs the single-tile plan redundantly in
// every workgroup and lets one of them write it out).
template <bool SINGLE, int R>
__device__ __forceinline__ void place_tile(PlaceLds<R> &s, const PlanArgs &a, int tile, bool writer)
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int tok0 = tile * a.tpt;
    const int ntok = min(a.tpt, a.N - tok0);
    const int npairs = ntok > 0 ? ntok * a.k : 0;
    const int64_t pair0 = (int64_t)tok0 * a.k;
    // experts and devices share one ranking pass when their bins fit the counters together
    const bool together = a.E + a.D <= kMaxBins;

    if (tid == 0) s.invalid = 0;
    __syncthreads();
    int ekey[R], tl[R];   // expert id and tile-local token of the thread's pairs
    int eraw[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int p = wave * (R * kWave) + r * kWave + lane;
        eraw[r] = p < npairs ? a.A[pair0 + p] : 0;
    }
    // counts of the other tiles: requested behind the routing, used after the ranking (see cross_prefetch)
    int cross[kCross];
    if constexpr (SINGLE) {
#pragma unroll
        for (int i = 0; i < kCross; ++i) cross[i] = 0;
    } else {
        cross_prefetch<kCross>(a, together ? a.E + a.D : a.E, 0, cross);
    }
    rank_clear(s, together ? a.E + a.D : a.E);   // while the loads are on their way
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int p = wave * (R * kWave) + r * kWave + lane;
        int key = -1;
        if (p < npairs) {
            const int e = eraw[r];
            if ((unsigned)e < (unsigned)a.E) key = e;
            else if constexpr (SINGLE) atomicAdd(&s.invalid, 1);
        }
        tl[r] = div20(p, a.k_magic);
        ekey[r] = key;
        s.tile_dev[p] = (int16_t)(key >= 0 ? div20(key, a.eloc_magic) : -1);
    }
    __syncthreads();

    // level 1: a token has one send row per device, taken at the device's first appearance among its entries
    const int dbits = bits_for(a.D);
    int dkey[R], jfirst[R];   // jfirst: the token's first pair on the same device
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int p = wave * (R * kWave) + r * kWave + lane;
        const int d = s.tile_dev[p];
        uint64_t same;
        jfirst[r] = first_pair_on_device(s.tile_dev, p, lane, tl[r] * a.k, d, dbits, same);
        dkey[r] = jfirst[r] == p ? d : -1;
    }

    // level 2 receive side (expert-major slot of every pair) and level 1 (send row of every first appearance)
    int slot[R], tile_pos[R], row[R];
    if (together) {
        int key2[2 * R], pos2[2 * R], tp2[2 * R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            key2[r] = ekey[r];
            key2[R + r] = dkey[r] >= 0 ? a.E + dkey[r] : -1;
        }
        rank_bins<SINGLE, R, 2 * R, kCross>(s, a, tile, writer, key2, a.E, a.D, 0, cross, pos2, tp2);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            slot[r] = pos2[r];
            tile_pos[r] = tp2[r];
            row[r] = pos2[R + r];
        }
    } else {
        int unused[R];
        rank_bins<SINGLE, R, R, kCross>(s, a, tile, writer, ekey, a.E, 0, 0, cross, slot, tile_pos);
        int cross_d[kCross];   // (the second pass has no expert bins and leaves s.tile_pairs alone)
        if constexpr (SINGLE) {
#pragma unroll
            for (int i = 0; i < kCross; ++i) cross_d[i] = 0;
        } else {
            cross_prefetch<kCross>(a, a.D, a.E, cross_d);
        }
        rank_clear(s, a.D);
        __syncthreads();
        rank_bins<SINGLE, R, R, kCross>(s, a, tile, writer, dkey, 0, a.D, a.E, cross_d, row, unused);
    }
    const int tile_pairs = s.tile_pairs;          // pairs of this tile with a valid expert id
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int p = wave * (R * kWave) + r * kWave + lane;
        s.tile_slot[p] = slot[r];
        if (writer && p < npairs) a.pair_slot[pair0 + p] = slot[r];
    }

    if (!writer) return;   // only the slots are wanted (uniform over the workgroup)

#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int p = wave * (R * kWave) + r * kWave + lane;
        s.tile_row[p] = row[r];
        if (p < npairs) {
            a.pair_first[pair0 + p] = row[r] >= 0 ? 1 : 0;
            if (row[r] >= 0) a.send_src[row[r]] = tok0 + tl[r];
        }
    }
    __syncthreads();

    // level 2 send side: every pair points at the send row of its token on its device
    int srow[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int p = wave * (R * kWave) + r * kWave + lane;
        srow[r] = ekey[r] >= 0 ? s.tile_row[jfirst[r]] : -1;
        if (p < npairs) a.pair_send_row[pair0 + p] = srow[r];
    }
    // The arrays indexed by slot are written in the tile's transfer order (its slots ascending: expert by expert,
    // tokens ascending), which is also the order that is listed for dispatch: neighbouring threads then write
    // neighbouring slots of one expert, a few cache lines per wave instead of 64.  The pairs meet their place in
    // that order through LDS; sorted_pair reuses the per-wave counters, which the ranking no longer needs.
    uint16_t *sorted_pair = &s.wave_cnt[0][0];
    static_assert(sizeof(s.wave_cnt) >= R * kRoundPairs * sizeof(uint16_t), "sorted_pair fits the per-wave counters");
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int p = wave * (R * kWave) + r * kWave + lane;
        if (tile_pos[r] >= 0) {
            sorted_pair[tile_pos[r]] = (uint16_t)p;
            // only pairs that are not a first appearance write here, and nobody reads their entry above
            if (jfirst[r] != p) s.tile_row[p] = srow[r];
        }
    }
    __syncthreads();
    const int cap = a.tpt * a.k;
    int32_t *order = a.tile_slots + (int64_t)tile * cap;
    for (int q = tid; q < cap; q += kPlanThreads) {
        if (q < tile_pairs) {
            const int p = sorted_pair[q];
            const int sl = s.tile_slot[p];
            order[q] = sl;
            a.slot_pair[sl] = (int32_t)(pair0 + p);
            a.slot_token[sl] = tok0 + div20(p, a.k_magic);
            a.slot_send_row[sl] = s.tile_row[p];
        } else {
            order[q] = -1;
        }
    }

    if (tile == 0 && wave == 0) {
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

template <bool SINGLE, int R>
__global__ __launch_bounds__(kPlanThreads) void plan_place_kernel(PlanArgs a)
{
    __shared__ PlaceLds<R> s;
    place_tile<SINGLE, R>(s, a, blockIdx.x, true);
}

// Cross-node traffic load of the GPU that owns this plan (section 3.4): bytes of the send rows whose
// destination device lies on another node than `home_node`.  One wave.
__global__ __launch_bounds__(kWave) void cross_node_load_kernel(const int32_t *send_count, int D, int devices_per_node,
                                                               int home_node, uint64_t row_bytes, int64_t *load)
{
    int64_t rows = 0;
    for (int d = threadIdx.x; d < D; d += kWave)
        if (d / devices_per_node != home_node) rows += send_count[d];
    for (int s = kWave / 2; s > 0; s >>= 1) rows += __shfl_down(rows, s, kWave);
    if (threadIdx.x == 0) *load = rows * (int64_t)row_bytes;
}

}   // namespace

#endif
