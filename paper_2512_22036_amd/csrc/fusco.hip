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

#include <stdint.h>
#include <stdlib.h>

#include "fusco.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;
constexpr int kPlanThreads = 256;                       // 4 waves per planner workgroup
constexpr int kPlanWaves = kPlanThreads / kWave;
constexpr int kTilePairs = 2048;                        // (token, expert) pairs per planner tile
constexpr int kRounds = kTilePairs / kPlanThreads;      // 64-pair rounds per wave
constexpr int kWaveChunk = kTilePairs / kPlanWaves;     // consecutive pairs owned by one wave
constexpr int kMaxBins = FUSCO_MAX_E;
constexpr size_t kMaxRowChunks = 1u << 16;              // rows of at most 1 MiB

static_assert(kTilePairs >= FUSCO_MAX_K, "a tile must hold at least one token");

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

bool sizes_ok(int32_t N, int32_t k, int32_t E, int32_t D)
{
    if (N < 0 || k < 1 || k > FUSCO_MAX_K || E < 1 || E > FUSCO_MAX_E || D < 1 || D > E) return false;
    if (E % D != 0) return false;
    if ((int64_t)N * k >= ((int64_t)1 << 31)) return false;
    return true;
}

inline int tokens_per_tile(int k) { return kTilePairs / k; }
inline int num_tiles(int N, int k)
{
    const int tpt = tokens_per_tile(k);
    const int n = (N + tpt - 1) / tpt;
    return n < 1 ? 1 : n;
}

// ------------------------------------------------------------------------------------------
// Planner
// ------------------------------------------------------------------------------------------
struct PlanArgs {
    const int32_t *A;
    int32_t N, k, E, D, Eloc;
    int32_t tpt;      // tokens per tile
    int32_t n_tiles;
    int32_t stride;   // ints per tile in tile_hist: E expert counts, D device counts, 1 invalid count
    int32_t *tile_hist;
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

// True iff pair (t_local, j) is the first entry of its token whose expert lives on device d.
__device__ __forceinline__ bool first_of_device(const int *tile_key, int row0, int j, int d, int Eloc)
{
    for (int j2 = 0; j2 < j; ++j2) {
        const int e2 = tile_key[row0 + j2];
        if (e2 >= 0 && e2 / Eloc == d) return false;
    }
    return true;
}

// Pass 1 of the multi-tile planner: per-tile counts of pairs per expert and of first
// (token, device) appearances per device.  Counts are order-independent, so LDS atomics are safe.
__global__ __launch_bounds__(kPlanThreads) void plan_count_kernel(PlanArgs a)
{
    __shared__ int tile_key[kTilePairs];
    __shared__ int hist[2 * kMaxBins + 1];
    const int tid = threadIdx.x;
    const int tile = blockIdx.x;
    const int tok0 = tile * a.tpt;
    const int ntok = min(a.tpt, a.N - tok0);
    const int npairs = ntok > 0 ? ntok * a.k : 0;
    const int64_t pair0 = (int64_t)tok0 * a.k;
    const int nb = a.E + a.D;

    for (int b = tid; b <= nb; b += kPlanThreads) hist[b] = 0;
    __syncthreads();
    for (int p = tid; p < npairs; p += kPlanThreads) {
        const int e = a.A[pair0 + p];
        int key = -1;
        if ((unsigned)e < (unsigned)a.E) {
            key = e;
            atomicAdd(&hist[e], 1);
        } else {
            atomicAdd(&hist[nb], 1);
        }
        tile_key[p] = key;
    }
    __syncthreads();
    for (int p = tid; p < npairs; p += kPlanThreads) {
        const int key = tile_key[p];
        if (key < 0) continue;
        const int tl = p / a.k, j = p - tl * a.k, d = key / a.Eloc;
        if (first_of_device(tile_key, tl * a.k, j, d, a.Eloc)) atomicAdd(&hist[a.E + d], 1);
    }
    __syncthreads();
    int32_t *out = a.tile_hist + (int64_t)tile * a.stride;
    for (int b = tid; b <= nb; b += kPlanThreads) out[b] = hist[b];
}

// Shared LDS state of the placement kernel.
struct PlaceLds {
    int tile_key[kTilePairs];
    int tile_slot[kTilePairs];
    int tile_row[kTilePairs];
    int wave_cnt[kPlanWaves][kMaxBins];
    int base[kMaxBins];
    int total[kMaxBins + 1];
    int invalid;
};

// Stable ranking of the tile's participating pairs by key, in pair order, on top of the global
// order of tiles.  key[r] is the key of pair (wave chunk + r * 64 + lane), or -1 if that pair
// does not take part.  On return pos[r] is the pair's global position: (global exclusive offset
// of its key) + (pairs with that key in earlier tiles) + (earlier pairs with that key in this
// tile).  Block 0 also writes the per-key counts and their exclusive prefix sum.
template <bool SINGLE>
__device__ __forceinline__ void rank_by_key(PlaceLds &s, const PlanArgs &a, const int (&key)[kRounds], int nb,
                                            int hist_off, int32_t *count_out, int32_t *off_out,
                                            int (&pos)[kRounds])
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int nbits = bits_for(nb);
    const uint64_t lt = ((uint64_t)1 << lane) - 1;

    for (int b = lane; b < nb; b += kWave) s.wave_cnt[wave][b] = 0;
    __syncthreads();

    // rank inside the wave's chunk; wave_cnt[wave][key] is the running count of the key
    int rank[kRounds];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const bool part = key[r] >= 0;
        const uint64_t m = same_key_lanes(key[r], part, nbits);
        const int before = part ? s.wave_cnt[wave][key[r]] : 0;
        rank[r] = before + __builtin_popcountll(m & lt);
        __syncthreads();
        if (part && (m & lt) == 0) s.wave_cnt[wave][key[r]] = before + __builtin_popcountll(m);
        __syncthreads();
    }

    // per key: total over all tiles and the part that lies in earlier tiles
    for (int b = tid; b < nb; b += kPlanThreads) {
        int tot = 0, pre = 0;
        if constexpr (SINGLE) {
            for (int w = 0; w < kPlanWaves; ++w) tot += s.wave_cnt[w][b];
        } else {
            const int32_t *h = a.tile_hist + hist_off + b;
            const int me = blockIdx.x;
            for (int tl = 0; tl < a.n_tiles; ++tl) {
                const int v = h[(int64_t)tl * a.stride];
                tot += v;
                pre += tl < me ? v : 0;
            }
        }
        s.total[b] = tot;
        s.base[b] = pre;
        if (blockIdx.x == 0) count_out[b] = tot;
    }
    __syncthreads();

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
    if (blockIdx.x == 0)
        for (int b = tid; b <= nb; b += kPlanThreads) off_out[b] = s.total[b];

    // turn the per-wave counts into per-wave starting positions
    for (int b = tid; b < nb; b += kPlanThreads) {
        int run = s.total[b] + s.base[b];
        for (int w = 0; w < kPlanWaves; ++w) {
            const int c = s.wave_cnt[w][b];
            s.wave_cnt[w][b] = run;
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRounds; ++r) pos[r] = key[r] >= 0 ? s.wave_cnt[wave][key[r]] + rank[r] : -1;
    __syncthreads();
}

// Pass 2 (or the only pass when the whole input is one tile): writes every descriptor array.
template <bool SINGLE>
__global__ __launch_bounds__(kPlanThreads) void plan_place_kernel(PlanArgs a)
{
    __shared__ PlaceLds s;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int tile = blockIdx.x;
    const int tok0 = tile * a.tpt;
    const int ntok = min(a.tpt, a.N - tok0);
    const int npairs = ntok > 0 ? ntok * a.k : 0;
    const int64_t pair0 = (int64_t)tok0 * a.k;

    if (tid == 0) s.invalid = 0;
    __syncthreads();
    int ekey[kRounds];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = wave * kWaveChunk + r * kWave + lane;
        int key = -1;
        if (p < npairs) {
            const int e = a.A[pair0 + p];
            if ((unsigned)e < (unsigned)a.E) key = e;
            else if constexpr (SINGLE) atomicAdd(&s.invalid, 1);
        }
        ekey[r] = key;
        s.tile_key[p] = key;
    }
    __syncthreads();

    // level 2 receive side: expert-major slot of every pair
    int slot[kRounds];
    rank_by_key<SINGLE>(s, a, ekey, a.E, 0, a.exp_count, a.exp_off, slot);
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = wave * kWaveChunk + r * kWave + lane;
        s.tile_slot[p] = slot[r];
        if (p < npairs) {
            a.pair_slot[pair0 + p] = slot[r];
            if (slot[r] >= 0) {
                a.slot_pair[slot[r]] = (int32_t)(pair0 + p);
                a.slot_token[slot[r]] = tok0 + p / a.k;
            }
        }
    }

    // level 1: one send row per (token, device), taken at the device's first appearance
    int dkey[kRounds];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = wave * kWaveChunk + r * kWave + lane;
        dkey[r] = -1;
        if (ekey[r] >= 0) {
            const int tl = p / a.k, j = p - tl * a.k, d = ekey[r] / a.Eloc;
            if (first_of_device(s.tile_key, tl * a.k, j, d, a.Eloc)) dkey[r] = d;
        }
    }
    int row[kRounds];
    rank_by_key<SINGLE>(s, a, dkey, a.D, a.E, a.send_count, a.send_off, row);
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = wave * kWaveChunk + r * kWave + lane;
        s.tile_row[p] = row[r];
        if (p < npairs) {
            a.pair_first[pair0 + p] = row[r] >= 0 ? 1 : 0;
            if (row[r] >= 0) a.send_src[row[r]] = tok0 + p / a.k;
        }
    }
    __syncthreads();

    // level 2 send side: every pair points at the send row of its token on its device
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = wave * kWaveChunk + r * kWave + lane;
        if (p >= npairs) continue;
        int srow = -1;
        if (ekey[r] >= 0) {
            const int tl = p / a.k, j = p - tl * a.k, d = ekey[r] / a.Eloc;
            int j0 = j;
            for (int j2 = 0; j2 < j; ++j2) {
                const int e2 = s.tile_key[tl * a.k + j2];
                if (e2 >= 0 && e2 / a.Eloc == d) { j0 = j2; break; }
            }
            srow = s.tile_row[tl * a.k + j0];
            a.slot_send_row[s.tile_slot[p]] = srow;
        }
        a.pair_send_row[pair0 + p] = srow;
    }

    if (blockIdx.x == 0 && tid == 0) {
        int bad = 0;
        if constexpr (SINGLE) bad = s.invalid;
        else
            for (int tl = 0; tl < a.n_tiles; ++tl) bad += a.tile_hist[(int64_t)tl * a.stride + a.E + a.D];
        *a.status = bad;
    }
}

// ------------------------------------------------------------------------------------------
// Dispatch: one workgroup column per token; the row is held in registers between the single
// read and the k (+ wire) writes.  Slot lookups depend only on blockIdx, so they are scalar.
// ------------------------------------------------------------------------------------------
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
        if (c < a.C) v[i] = __builtin_nontemporal_load(a.x + (size_t)t * a.C + c);
        else if (c < Ct) v[i] = __builtin_nontemporal_load(a.x_aux + (size_t)t * a.Ca + (c - a.C));
    }
    const int32_t *slots = a.pair_slot + (size_t)t * a.k;
    if (a.write_expert) {
        for (int j = 0; j < a.k; ++j) {
            const int slot = slots[j];
            if (slot < 0) continue;
#pragma unroll
            for (int i = 0; i < CPT; ++i) {
                const int c = c0 + i * blockDim.x;
                if (c < a.C) __builtin_nontemporal_store(v[i], a.expert_buf + (size_t)slot * a.C + c);
                else if (c < Ct) __builtin_nontemporal_store(v[i], a.expert_aux + (size_t)slot * a.Ca + (c - a.C));
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
                if (c < a.C) __builtin_nontemporal_store(v[i], a.send_buf + (size_t)row * a.C + c);
                else if (c < Ct) __builtin_nontemporal_store(v[i], a.send_aux + (size_t)row * a.Ca + (c - a.C));
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Combine: one workgroup column per token; every thread owns CPT 16-byte chunks of the output
// row, pulls the matching chunks of the token's k rows (JU rows in flight at a time) and
// accumulates in fp32 with one fused multiply-add per term in ascending j.
// ------------------------------------------------------------------------------------------
struct CombineArgs {
    const u32x4 *y;
    const float *w;
    void *out;
    const int32_t *pair_slot;
    int32_t k;
    int32_t C;   // 16-byte chunks per y row
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

template <bool Y_BF16, bool OUT_BF16, int CPT, int JU>
__global__ __launch_bounds__(256) void combine_kernel(CombineArgs a)
{
    constexpr int EPC = Y_BF16 ? 8 : 4;   // elements per 16-byte chunk of y
    const int t = blockIdx.x;
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
                if (slot >= 0) {
                    on[jj] = true;
#pragma unroll
                    for (int i = 0; i < CPT; ++i) {
                        const int c = c0 + i * blockDim.x;
                        if (c < a.C) v[jj][i] = __builtin_nontemporal_load(a.y + (size_t)slot * a.C + c);
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
        const size_t e0 = ((size_t)t * a.C + c) * EPC;   // first output element of this chunk
        if constexpr (OUT_BF16) {
            uint32_t pk[EPC / 2];
#pragma unroll
            for (int q = 0; q < EPC / 2; ++q) pk[q] = to_bf16(acc[i][2 * q]) | (to_bf16(acc[i][2 * q + 1]) << 16);
            if constexpr (Y_BF16) {
                u32x4 o = {pk[0], pk[1], pk[2], pk[3]};
                __builtin_nontemporal_store(o, (u32x4 *)((uint16_t *)a.out + e0));
            } else {
                u32x2 o = {pk[0], pk[1]};
                __builtin_nontemporal_store(o, (u32x2 *)((uint16_t *)a.out + e0));
            }
        } else {
#pragma unroll
            for (int h = 0; h < EPC / 4; ++h) {
                u32x4 o = {__float_as_uint(acc[i][4 * h]), __float_as_uint(acc[i][4 * h + 1]),
                           __float_as_uint(acc[i][4 * h + 2]), __float_as_uint(acc[i][4 * h + 3])};
                __builtin_nontemporal_store(o, (u32x4 *)((float *)a.out + e0) + h);
            }
        }
    }
}


// ---- experimental movers (selected through environment variables while tuning) -------------
struct XArgs {
    DispatchArgs d;
    const int32_t *slot_token, *exp_off, *send_src, *send_off;
    int32_t E, D, N;
    int32_t S;      // 64-chunk segments per row
    int32_t WPT;    // waves per row
    int32_t nt;     // bit 0: non-temporal loads, bit 1: non-temporal stores
};

__device__ __forceinline__ u32x4 ld16(const u32x4 *p, bool nt) { return nt ? __builtin_nontemporal_load(p) : *p; }
__device__ __forceinline__ void st16(u32x4 v, u32x4 *p, bool nt)
{
    if (nt) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// token-major, wave-centric: a wave owns UPW consecutive 64-chunk segments of one token row
template <int UPW>
__global__ __launch_bounds__(256) void dispatch_wave_kernel(XArgs a)
{
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + (threadIdx.x >> 6));
    const int t = w / a.WPT;
    if (t >= a.N) return;
    const int seg0 = (w - t * a.WPT) * UPW;
    const int C = a.d.C, Ca = a.d.Ca, Ct = C + Ca;
    const bool ntl = a.nt & 1, nts = a.nt & 2;
    u32x4 v[UPW];
#pragma unroll
    for (int i = 0; i < UPW; ++i) {
        const int c = (seg0 + i) * 64 + lane;
        if (c < C) v[i] = ld16(a.d.x + (size_t)t * C + c, ntl);
        else if (c < Ct) v[i] = ld16(a.d.x_aux + (size_t)t * Ca + (c - C), ntl);
    }
    const int32_t *slots = a.d.pair_slot + (size_t)t * a.d.k;
    if (a.d.write_expert) {
        for (int j = 0; j < a.d.k; ++j) {
            const int slot = slots[j];
            if (slot < 0) continue;
#pragma unroll
            for (int i = 0; i < UPW; ++i) {
                const int c = (seg0 + i) * 64 + lane;
                if (c < C) st16(v[i], a.d.expert_buf + (size_t)slot * C + c, nts);
                else if (c < Ct) st16(v[i], a.d.expert_aux + (size_t)slot * Ca + (c - C), nts);
            }
        }
    }
    if (a.d.write_wire) {
        const int32_t *rows = a.d.pair_send_row + (size_t)t * a.d.k;
        const uint8_t *first = a.d.pair_first + (size_t)t * a.d.k;
        for (int j = 0; j < a.d.k; ++j) {
            if (!first[j]) continue;
            const int row = rows[j];
#pragma unroll
            for (int i = 0; i < UPW; ++i) {
                const int c = (seg0 + i) * 64 + lane;
                if (c < C) st16(v[i], a.d.send_buf + (size_t)row * C + c, nts);
                else if (c < Ct) st16(v[i], a.d.send_aux + (size_t)row * Ca + (c - C), nts);
            }
        }
    }
}

// destination-major: a wave owns UPW consecutive segments of one destination row and pulls
// them from the source token row; destination rows are written in address order
template <int UPW, bool WIRE>
__global__ __launch_bounds__(256) void dispatch_rows_kernel(XArgs a)
{
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + (threadIdx.x >> 6));
    const int r = w / a.WPT;
    const int nrows = WIRE ? a.send_off[a.D] : a.exp_off[a.E];
    if (r >= nrows) return;
    const int t = WIRE ? a.send_src[r] : a.slot_token[r];
    const int seg0 = (w - r * a.WPT) * UPW;
    const int C = a.d.C, Ca = a.d.Ca, Ct = C + Ca;
    const bool ntl = a.nt & 1, nts = a.nt & 2;
    u32x4 *dst = WIRE ? a.d.send_buf : a.d.expert_buf;
    u32x4 *dst_aux = WIRE ? a.d.send_aux : a.d.expert_aux;
    u32x4 v[UPW];
#pragma unroll
    for (int i = 0; i < UPW; ++i) {
        const int c = (seg0 + i) * 64 + lane;
        if (c < C) v[i] = ld16(a.d.x + (size_t)t * C + c, ntl);
        else if (c < Ct) v[i] = ld16(a.d.x_aux + (size_t)t * Ca + (c - C), ntl);
    }
#pragma unroll
    for (int i = 0; i < UPW; ++i) {
        const int c = (seg0 + i) * 64 + lane;
        if (c < C) st16(v[i], dst + (size_t)r * C + c, nts);
        else if (c < Ct) st16(v[i], dst_aux + (size_t)r * Ca + (c - C), nts);
    }
}

int env_int(const char *name, int dflt)
{
    const char *s = getenv(name);
    return s ? atoi(s) : dflt;
}

__global__ __launch_bounds__(256) void probe_copy_kernel(u32x4 *dst, const u32x4 *src, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

int round_up(int v, int m) { return (v + m - 1) / m * m; }

// Optional launch-shape override for tuning runs: "<threads>,<chunks per thread>".
bool shape_from_env(const char *name, int *threads, int *cpt)
{
    const char *s = getenv(name);
    if (!s) return false;
    char *end = nullptr;
    const long th = strtol(s, &end, 10);
    if (!end || *end != ',') return false;
    const long cp = strtol(end + 1, nullptr, 10);
    if (th < 64 || th > 256 || th % 64 != 0) return false;
    if (cp != 1 && cp != 2 && cp != 4) return false;
    *threads = (int)th;
    *cpt = (int)cp;
    return true;
}

int launch_status()
{
    return hipGetLastError() == hipSuccess ? FUSCO_OK : FUSCO_ERR_HIP;
}

template <bool Y_BF16, bool OUT_BF16>
void launch_combine(const CombineArgs &a, int N, int threads, int cpt, hipStream_t s)
{
    const int segs = (a.C + threads * cpt - 1) / (threads * cpt);
    const dim3 grid((unsigned)N, (unsigned)segs), block((unsigned)threads);
    if (cpt == 1) hipLaunchKernelGGL((combine_kernel<Y_BF16, OUT_BF16, 1, 8>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((combine_kernel<Y_BF16, OUT_BF16, 2, 8>), grid, block, 0, s, a);
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
    return align_up((size_t)num_tiles(N, k) * (size_t)(E + D + 1) * 4, 256);
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

int fusco_plan(fusco_layout *L, const int32_t *d_topk_idx, void *d_scratch, size_t scratch_bytes, void *stream)
{
    if (!layout_ok(L) || (!d_topk_idx && L->N > 0) || !d_scratch) return FUSCO_ERR_INVALID_ARG;
    if (scratch_bytes < fusco_scratch_bytes(L->N, L->k, L->E, L->D)) return FUSCO_ERR_WORKSPACE;
    PlanArgs a;
    a.A = d_topk_idx;
    a.N = L->N; a.k = L->k; a.E = L->E; a.D = L->D; a.Eloc = L->E / L->D;
    a.tpt = tokens_per_tile(L->k);
    a.n_tiles = num_tiles(L->N, L->k);
    a.stride = L->E + L->D + 1;
    a.tile_hist = (int32_t *)d_scratch;
    a.exp_count = L->exp_count; a.exp_off = L->exp_off; a.send_count = L->send_count; a.send_off = L->send_off;
    a.pair_slot = L->pair_slot; a.slot_pair = L->slot_pair; a.slot_token = L->slot_token; a.send_src = L->send_src;
    a.pair_send_row = L->pair_send_row; a.slot_send_row = L->slot_send_row; a.pair_first = L->pair_first;
    a.status = L->status;
    hipStream_t s = (hipStream_t)stream;
    if (a.n_tiles == 1) {
        hipLaunchKernelGGL(plan_place_kernel<true>, dim3(1), dim3(kPlanThreads), 0, s, a);
    } else {
        hipLaunchKernelGGL(plan_count_kernel, dim3(a.n_tiles), dim3(kPlanThreads), 0, s, a);
        hipLaunchKernelGGL(plan_place_kernel<false>, dim3(a.n_tiles), dim3(kPlanThreads), 0, s, a);
    }
    return launch_status();
}

int fusco_dispatch(const fusco_layout *L, const void *d_x, size_t row_bytes, const void *d_x_aux,
                   size_t aux_row_bytes, void *d_expert_buf, void *d_expert_aux, void *d_send_buf,
                   void *d_send_aux, uint32_t flags, void *stream)
{
    if (!layout_ok(L) || !d_x) return FUSCO_ERR_INVALID_ARG;
    if (flags == 0) flags = FUSCO_DISPATCH_EXPERT;
    if (flags & ~(FUSCO_DISPATCH_EXPERT | FUSCO_DISPATCH_WIRE)) return FUSCO_ERR_UNSUPPORTED;
    const bool expert = flags & FUSCO_DISPATCH_EXPERT, wire = flags & FUSCO_DISPATCH_WIRE;
    if (row_bytes == 0 || row_bytes % 16 != 0 || aux_row_bytes % 16 != 0) return FUSCO_ERR_INVALID_ARG;
    if ((row_bytes + aux_row_bytes) / 16 > kMaxRowChunks) return FUSCO_ERR_INVALID_ARG;
    if (aux_row_bytes && !d_x_aux) return FUSCO_ERR_INVALID_ARG;
    if (expert && (!d_expert_buf || (aux_row_bytes && !d_expert_aux))) return FUSCO_ERR_INVALID_ARG;
    if (wire && (!d_send_buf || (aux_row_bytes && !d_send_aux))) return FUSCO_ERR_INVALID_ARG;
    if (!aligned16(d_x) || !aligned16(d_x_aux) || !aligned16(d_expert_buf) || !aligned16(d_expert_aux) ||
        !aligned16(d_send_buf) || !aligned16(d_send_aux))
        return FUSCO_ERR_INVALID_ARG;
    if (L->N == 0) return FUSCO_OK;

    DispatchArgs a;
    a.x = (const u32x4 *)d_x;
    a.x_aux = (const u32x4 *)d_x_aux;
    a.expert_buf = (u32x4 *)d_expert_buf; a.expert_aux = (u32x4 *)d_expert_aux;
    a.send_buf = (u32x4 *)d_send_buf; a.send_aux = (u32x4 *)d_send_aux;
    a.pair_slot = L->pair_slot; a.pair_send_row = L->pair_send_row; a.pair_first = L->pair_first;
    a.k = L->k;
    a.C = (int32_t)(row_bytes / 16);
    a.Ca = (int32_t)(aux_row_bytes / 16);
    a.write_expert = expert; a.write_wire = wire;
    const int Ct = a.C + a.Ca;

    const int mode = env_int("FUSCO_DISPATCH_MODE", 0);
    if (mode != 0) {
        XArgs xa;
        xa.d = a;
        xa.slot_token = L->slot_token; xa.exp_off = L->exp_off; xa.send_src = L->send_src; xa.send_off = L->send_off;
        xa.E = L->E; xa.D = L->D; xa.N = L->N;
        xa.S = (Ct + 63) / 64;
        int upw = env_int("FUSCO_UPW", 2);
        if (upw != 1 && upw != 2 && upw != 4) upw = 2;
        xa.WPT = (xa.S + upw - 1) / upw;
        xa.nt = env_int("FUSCO_NT", 3);
        hipStream_t s = (hipStream_t)stream;
        if (mode == 1) {
            const int64_t waves = (int64_t)L->N * xa.WPT;
            const dim3 grid((unsigned)((waves + 3) / 4)), block(256);
            if (upw == 1) hipLaunchKernelGGL(dispatch_wave_kernel<1>, grid, block, 0, s, xa);
            else if (upw == 2) hipLaunchKernelGGL(dispatch_wave_kernel<2>, grid, block, 0, s, xa);
            else hipLaunchKernelGGL(dispatch_wave_kernel<4>, grid, block, 0, s, xa);
        } else {
            if (expert) {
                xa.N = L->P;
                const int64_t waves = (int64_t)L->P * xa.WPT;
                const dim3 grid((unsigned)((waves + 3) / 4)), block(256);
                if (upw == 1) hipLaunchKernelGGL((dispatch_rows_kernel<1, false>), grid, block, 0, s, xa);
                else if (upw == 2) hipLaunchKernelGGL((dispatch_rows_kernel<2, false>), grid, block, 0, s, xa);
                else hipLaunchKernelGGL((dispatch_rows_kernel<4, false>), grid, block, 0, s, xa);
            }
            if (wire) {
                const int64_t waves = (int64_t)L->send_cap * xa.WPT;
                const dim3 grid((unsigned)((waves + 3) / 4)), block(256);
                if (upw == 1) hipLaunchKernelGGL((dispatch_rows_kernel<1, true>), grid, block, 0, s, xa);
                else if (upw == 2) hipLaunchKernelGGL((dispatch_rows_kernel<2, true>), grid, block, 0, s, xa);
                else hipLaunchKernelGGL((dispatch_rows_kernel<4, true>), grid, block, 0, s, xa);
            }
        }
        return launch_status();
    }
    int cpt = Ct >= 512 ? 4 : (Ct >= 128 ? 2 : 1);
    int threads = round_up((Ct + cpt - 1) / cpt, kWave);
    if (threads > 256) threads = 256;
    shape_from_env("FUSCO_DISPATCH_SHAPE", &threads, &cpt);
    const int segs = (Ct + threads * cpt - 1) / (threads * cpt);
    const dim3 grid((unsigned)L->N, (unsigned)segs), block((unsigned)threads);
    hipStream_t s = (hipStream_t)stream;
    switch (cpt) {
    case 1: hipLaunchKernelGGL(dispatch_kernel<1>, grid, block, 0, s, a); break;
    case 2: hipLaunchKernelGGL(dispatch_kernel<2>, grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL(dispatch_kernel<4>, grid, block, 0, s, a); break;
    }
    return launch_status();
}

int fusco_combine(const fusco_layout *L, const void *d_y, int y_dtype, const float *d_w, void *d_out,
                  int out_dtype, int32_t H, uint32_t flags, void *stream)
{
    if (!layout_ok(L) || !d_y || !d_w || !d_out || H <= 0) return FUSCO_ERR_INVALID_ARG;
    if (flags != 0) return FUSCO_ERR_UNSUPPORTED;
    if ((y_dtype != FUSCO_BF16 && y_dtype != FUSCO_F32) || (out_dtype != FUSCO_BF16 && out_dtype != FUSCO_F32))
        return FUSCO_ERR_UNSUPPORTED;
    const size_t y_row = (size_t)H * (y_dtype == FUSCO_BF16 ? 2 : 4);
    if (y_row % 16 != 0 || y_row / 16 > kMaxRowChunks) return FUSCO_ERR_INVALID_ARG;
    if (!aligned16(d_y) || !aligned16(d_out) || ((uintptr_t)d_w & 3u)) return FUSCO_ERR_INVALID_ARG;
    if (L->N == 0) return FUSCO_OK;

    CombineArgs a;
    a.y = (const u32x4 *)d_y;
    a.w = d_w;
    a.out = d_out;
    a.pair_slot = L->pair_slot;
    a.k = L->k;
    a.C = (int32_t)(y_row / 16);
    int cpt = 1;
    int threads = round_up(a.C, kWave);
    if (threads > 256) threads = 256;
    shape_from_env("FUSCO_COMBINE_SHAPE", &threads, &cpt);
    if (cpt > 2) cpt = 2;
    hipStream_t s = (hipStream_t)stream;
    if (y_dtype == FUSCO_BF16 && out_dtype == FUSCO_BF16) launch_combine<true, true>(a, L->N, threads, cpt, s);
    else if (y_dtype == FUSCO_BF16) launch_combine<true, false>(a, L->N, threads, cpt, s);
    else if (out_dtype == FUSCO_BF16) launch_combine<false, true>(a, L->N, threads, cpt, s);
    else launch_combine<false, false>(a, L->N, threads, cpt, s);
    return launch_status();
}

int fusco_probe_copy(void *d_dst, const void *d_src, size_t bytes, void *stream)
{
    if (!d_dst || !d_src || bytes % 16 != 0 || !aligned16(d_dst) || !aligned16(d_src)) return FUSCO_ERR_INVALID_ARG;
    if (bytes == 0) return FUSCO_OK;
    const size_t n = bytes / 16;
    size_t blocks = (n + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(probe_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       (u32x4 *)d_dst, (const u32x4 *)d_src, n);
    return launch_status();
}

}   // extern "C"
