// Types, limits and small host helpers shared by every part of the library (one translation unit).
#ifndef FUSCO_CSRC_COMMON_H
#define FUSCO_CSRC_COMMON_H

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

}   // namespace

#endif
