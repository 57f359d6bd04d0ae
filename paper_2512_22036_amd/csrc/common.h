// Types, limits and small host helpers shared by every part of the library (one translation unit).
#ifndef FUSCO_CSRC_COMMON_H
#define FUSCO_CSRC_COMMON_H

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stdlib.h>
#include "fusco.h"
#include "fusco_probe.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;
constexpr int kPlanThreads = 1024;                      // 16 waves per planner workgroup
constexpr int kPlanWaves = kPlanThreads / kWave;
// A planner tile holds R * 1024 (token, expert) pairs, R rounds of 64 pairs per wave: one round for inputs of
// up to 1024 pairs, two otherwise.  (Four would not fit 64 KiB of LDS.)
constexpr int kMaxRounds = 2;
constexpr int kRoundPairs = kPlanThreads;               // pairs of one round of the whole workgroup
constexpr int kMaxBins = FUSCO_MAX_E;
constexpr size_t kMaxRowChunks = FUSCO_MAX_ROW_BYTES / 16;

static_assert(kRoundPairs >= FUSCO_MAX_K, "a tile must hold at least one token");
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
// Measured: with one round per tile the extra launch pays from about 320 tiles, with two rounds from 96.
inline int chunk_min_tiles(int rounds) { return rounds == 1 ? 320 : 96; }

inline int tokens_per_tile(int k, int rounds) { return rounds * kRoundPairs / k; }
inline int num_tiles(int N, int k, int rounds)
{
    const int tpt = tokens_per_tile(k, rounds);
    const int n = (N + tpt - 1) / tpt;
    return n < 1 ? 1 : n;
}

// Rounds with which the whole input is one tile (single-launch planner, fused plan + dispatch), or 0.
inline int single_tile_rounds(int N, int k)
{
    for (int r = 1; r <= kMaxRounds; r *= 2)
        if (N <= tokens_per_tile(k, r)) return r;
    return 0;
}

// Rounds per tile of the planner for these sizes.  A tile is also the unit in which dispatch moves rows
// (expert by expert inside a tile): two rounds give every expert twice as many neighbouring rows per tile,
// which is worth more to dispatch (5 us at 8192 tokens x 8) than the 2-3 us the planner loses against one round.
inline int plan_rounds(int N, int k)
{
    const int single = single_tile_rounds(N, k);
    return single ? single : kMaxRounds;
}

// tiles per chunk (a power of two near sqrt(n_tiles)), or 0 when the tiles are few enough to be read one by one
inline int chunk_tiles_for(int n_tiles, int rounds)
{
    if (n_tiles < chunk_min_tiles(rounds)) return 0;
    int c = 8;
    while (c * c < n_tiles) c *= 2;
    return c;
}
inline int num_chunks(int n_tiles, int rounds)
{
    const int c = chunk_tiles_for(n_tiles, rounds);
    return c ? (n_tiles + c - 1) / c : 0;
}

}   // namespace

#endif
