// MoE token shuffle with fused layout transformation for MI355X (gfx950, wave64).
//
// Three groups of kernels behind the C boundary declared in fusco.h:
//   planner  - token-expert matrix -> two-level layout descriptor (paper section 3.3)
//   dispatch - read every token row once, store it to all of its final rows (section 3.2)
//   combine  - per token, gather its k expert-output rows, weighted fp32 sum, one row out
// The path is pure data movement (no dense contraction), so there is no MFMA here: the movers
// are built around 16-byte coalesced global accesses, the planner around LDS counters and
// wave64 ballots.
//
// One translation unit: the kernels live in the headers next to this file (planner.h, movers.h,
// segments.h, probes.h), the host-side helpers in launch.h, the C entry points below.
#include "launch.h"
#include <atomic>
#include <mutex>

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
    case FUSCO_ERR_STATIC_LIMIT: return "input needs more planner scratch than the library's static buffer holds";
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
    const int rounds = plan_rounds(N, k);
    const int tile_tokens = tokens_per_tile(k, rounds), tile_count = num_tiles(N, k, rounds);
    int32_t *tile_slots = (int32_t *)take((size_t)tile_count * (size_t)tile_tokens * (size_t)k * 4);
    if (L) {
        L->N = N; L->k = k; L->E = E; L->D = D; L->P = (int32_t)P; L->send_cap = (int32_t)send_cap;
        L->exp_count = exp_count; L->exp_off = exp_off; L->send_count = send_count; L->send_off = send_off;
        L->status = status; L->pair_slot = pair_slot; L->slot_pair = slot_pair; L->slot_token = slot_token;
        L->send_src = send_src; L->pair_send_row = pair_send_row; L->slot_send_row = slot_send_row;
        L->pair_first = pair_first;
        L->tile_slots = tile_slots; L->tile_tokens = tile_tokens; L->tile_count = tile_count;
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
    const int rounds = plan_rounds(N, k);
    const int tiles = num_tiles(N, k, rounds);
    return align_up(((size_t)tiles + (size_t)num_chunks(tiles, rounds)) * (size_t)(E + D + 1) * 4, 256);
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
    const int rounds = plan_rounds(L->N, L->k);
    if (L->tile_tokens != tokens_per_tile(L->k, rounds) || L->tile_count != num_tiles(L->N, L->k, rounds)) return false;
    return L->exp_count && L->exp_off && L->send_count && L->send_off && L->pair_slot && L->slot_pair &&
           L->slot_token && L->send_src && L->pair_send_row && L->slot_send_row && L->pair_first && L->status &&
           L->tile_slots;
}

static PlanArgs plan_args(const fusco_layout *L, const int32_t *d_topk_idx, void *d_scratch, int rounds)
{
    PlanArgs a;
    a.A = d_topk_idx;
    a.N = L->N; a.k = L->k; a.E = L->E; a.D = L->D; a.Eloc = L->E / L->D;
    a.k_magic = ((1u << 20) + a.k - 1) / a.k;
    a.eloc_magic = ((1u << 20) + a.Eloc - 1) / a.Eloc;
    a.tpt = tokens_per_tile(L->k, rounds);
    a.n_tiles = num_tiles(L->N, L->k, rounds);
    a.stride = L->E + L->D + 1;
    a.tile_hist = (int32_t *)d_scratch;   // unused (may be NULL) when the input is a single tile
    a.chunk_tiles = chunk_tiles_for(a.n_tiles, rounds);
    a.n_chunks = num_chunks(a.n_tiles, rounds);
    a.chunk_hist = a.tile_hist + (size_t)a.n_tiles * (size_t)a.stride;
    a.exp_count = L->exp_count; a.exp_off = L->exp_off; a.send_count = L->send_count; a.send_off = L->send_off;
    a.pair_slot = L->pair_slot; a.slot_pair = L->slot_pair; a.slot_token = L->slot_token; a.send_src = L->send_src;
    a.pair_send_row = L->pair_send_row; a.slot_send_row = L->slot_send_row; a.pair_first = L->pair_first;
    a.tile_slots = L->tile_slots;
    a.status = L->status;
    return a;
}

int fusco_plan(fusco_layout *L, const int32_t *d_topk_idx, void *d_scratch, size_t scratch_bytes, void *stream)
{
    if (!layout_ok(L) || (!d_topk_idx && L->N > 0) || !d_scratch) return FUSCO_ERR_INVALID_ARG;
    if (scratch_bytes < fusco_scratch_bytes(L->N, L->k, L->E, L->D)) return FUSCO_ERR_WORKSPACE;
    const int rounds = plan_rounds(L->N, L->k);
    const PlanArgs a = plan_args(L, d_topk_idx, d_scratch, rounds);
    hipStream_t s = (hipStream_t)stream;
    const ArmedEvents ev;
    const dim3 block(kPlanThreads), tiles((unsigned)a.n_tiles);
    if (a.n_tiles == 1) {
        if (rounds == 1) launch(plan_place_kernel<true, 1>, dim3(1), block, s, a, ev.start, ev.stop);
        else launch(plan_place_kernel<true, 2>, dim3(1), block, s, a, ev.start, ev.stop);
    } else {
        // inputs of several tiles are always planned in tiles of two rounds (plan_rounds)
        launch(plan_count_kernel<kMaxRounds>, tiles, block, s, a, ev.start, nullptr);
        if (a.n_chunks > 0) launch(plan_chunk_kernel, dim3((unsigned)a.n_chunks), block, s, a);
        launch(plan_place_kernel<false, kMaxRounds>, tiles, block, s, a, nullptr, ev.stop);
    }
    return launch_status();
}

// Planner scratch that belongs to the library, for fusco_plan_static.  In host code the array's name is
// only a handle: the device address is looked up once per device with hipGetSymbolAddress and kept.
static __device__ __align__(256) unsigned char g_static_scratch[FUSCO_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void *g_static_scratch_ptr[kMaxDevices];   // per device: address of that GPU's copy of the array, or null
std::mutex g_static_scratch_lock;

// Device address of the calling thread's current GPU's copy of g_static_scratch, or null on failure.
void *static_scratch_of_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> hold(g_static_scratch_lock);
    if (!g_static_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_static_scratch_ptr[dev] = p;
    }
    return g_static_scratch_ptr[dev];
}
}   // namespace

int fusco_plan_static(fusco_layout *L, const int32_t *d_topk_idx, void *stream)
{
    if (!layout_ok(L) || (!d_topk_idx && L->N > 0)) return FUSCO_ERR_INVALID_ARG;
    if (fusco_scratch_bytes(L->N, L->k, L->E, L->D) > FUSCO_STATIC_SCRATCH_BYTES) return FUSCO_ERR_STATIC_LIMIT;
    void *scratch = static_scratch_of_current_device();
    if (!scratch) return FUSCO_ERR_HIP;
    // the planner writes every count it later reads, so the array needs no clearing between calls
    return fusco_plan(L, d_topk_idx, scratch, FUSCO_STATIC_SCRATCH_BYTES, stream);
}

int fusco_plan_dispatch(fusco_layout *L, const int32_t *d_topk_idx, const void *d_x, size_t row_bytes,
                        const void *d_x_aux, size_t aux_row_bytes, void *d_expert_buf, void *d_expert_aux,
                        void *stream)
{
    if (!layout_ok(L) || (!d_topk_idx && L->N > 0)) return FUSCO_ERR_INVALID_ARG;
    if (row_bytes == 0 || row_bytes % 16 != 0 || aux_row_bytes % 16 != 0) return FUSCO_ERR_INVALID_ARG;
    if ((row_bytes + aux_row_bytes) / 16 > kMaxRowChunks) return FUSCO_ERR_INVALID_ARG;
    const int rounds = single_tile_rounds(L->N, L->k);
    if (rounds == 0) return FUSCO_ERR_UNSUPPORTED;
    if (L->N > 0) {
        if (!d_x || !d_expert_buf || (aux_row_bytes && (!d_x_aux || !d_expert_aux))) return FUSCO_ERR_INVALID_ARG;
        if (!aligned16(d_x) || !aligned16(d_x_aux) || !aligned16(d_expert_buf) || !aligned16(d_expert_aux))
            return FUSCO_ERR_INVALID_ARG;
    }
    const PlanArgs a = plan_args(L, d_topk_idx, nullptr, rounds);
    DispatchArgs m;
    m.x = (const u32x4 *)d_x; m.x_aux = (const u32x4 *)d_x_aux;
    m.expert_buf = (u32x4 *)d_expert_buf; m.expert_aux = (u32x4 *)d_expert_aux;
    m.send_buf = nullptr; m.send_aux = nullptr;
    m.pair_slot = L->pair_slot; m.pair_send_row = L->pair_send_row; m.pair_first = L->pair_first;
    m.slot_token = nullptr; m.tile_slots = nullptr; m.tile_cap = 0; m.tile_tokens = 0; m.N = L->N; m.segs = 1; m.seg_chunks = 0;
    m.k = L->k;
    m.C = (int32_t)(row_bytes / 16); m.Ca = (int32_t)(aux_row_bytes / 16);
    m.write_expert = 1; m.write_wire = 0;
    const ArmedEvents ev;
    const dim3 grid((unsigned)(L->N > 0 ? L->N : 1)), block(kPlanThreads);
    hipStream_t s = (hipStream_t)stream;
    if (ev.start || ev.stop) {
        if (rounds == 1) hipExtLaunchKernelGGL(plan_dispatch_kernel<1>, grid, block, 0, s, ev.start, ev.stop, 0, a, m);
        else hipExtLaunchKernelGGL(plan_dispatch_kernel<2>, grid, block, 0, s, ev.start, ev.stop, 0, a, m);
    } else {
        if (rounds == 1) hipLaunchKernelGGL(plan_dispatch_kernel<1>, grid, block, 0, s, a, m);
        else hipLaunchKernelGGL(plan_dispatch_kernel<2>, grid, block, 0, s, a, m);
    }
    return launch_status();
}

// largest source tensor that the tiled dispatch takes in one piece (fusco_probe_source_chunk_bytes changes it)
static std::atomic<size_t> g_source_chunk_bytes{kSourceChunkBytes};

// fusco_probe_dispatch_kernel: 0 automatic; 1 keeps fusco_dispatch on the token walk; 2 takes the transfer order
// wherever its shape allows, whatever the sizes (for comparisons and tests)
static std::atomic<int> g_dispatch_kernel{0};

// fusco_probe_dispatch_occupancy: workgroups of the tiled dispatch per compute unit; 0 automatic
static std::atomic<int> g_tiled_occupancy{0};

// fusco_probe_dispatch_walk: 0 automatic; 1 + (bit 0 cached loads, bit 1 non-temporal stores)
static std::atomic<int> g_walk_mode{0};

// fusco_probe_dispatch_pull: 0 automatic, 1 off, 2 on
static std::atomic<int> g_tiled_pull{0};

// Dynamic LDS that lets `wgs` workgroups share a compute unit's 160 KiB of LDS, which is handed out in 128 blocks
// of 1280 bytes (3 <= wgs <= 15; 13 comes out as 14; the kernels have no LDS of their own); 0 for no cap.
static size_t lds_for_occupancy(int wgs)
{
    if (wgs < 3 || wgs > 15) return 0;
    return (size_t)(128 / wgs) * 1280;
}

// Workgroups of the tiled dispatch per compute unit for rows (or column segments) of seg_bytes, source tensor
// resident in the memory-side cache (16: no cap).  The kernel runs at the rate of its writes, which is higher the
// fewer rows are being written at a time, as long as enough loads stay in flight: about 70-90 KiB of rows per compute
// unit.  Measured at 8192 tokens x 8, dispatch alone, us, no cap / the cap chosen / one less: 5 KiB rows 66.6 /
// 58.6 (12) / 58.9; 6 KiB 75.5 / 71.5 (12) / 71.7; 8 KiB 96.2 / 87.2 (12) / 87.8; 10 KiB 118.6 / 111.5 (8) / 113.8;
// 12 KiB 140.2 / 131.9 (7) / 140.1; 13 KiB 151 / 146 (6) / 149; 14 KiB 165 / 157 (5) / 171; 15 KiB 173 / 164 (5) / 177;
// two segments of 8 KiB 192.1 / 189.3 (12); of 12 KiB (4096 tokens) 142.2 / 135.1 (7).  Rows shorter than 4 KiB
// are moved by workgroups of one or two waves, of which a compute unit should hold more than a cap allows.
static int tiled_workgroups_per_cu(size_t seg_bytes)
{
    if (seg_bytes < 4096) return 16;
    if (seg_bytes <= 8192) return 12;
    if (seg_bytes <= 10240) return 8;
    if (seg_bytes <= 12288) return 7;
    if (seg_bytes <= 13312) return 6;
    return 5;
}

// Workgroup shape of the tiled dispatch for rows of Ct 16-byte chunks (both planes): the rows are cut into
// `segs` column segments of `per` chunks, a tile being worked through once per segment, so that the segment
// of the tile's source rows that is in use fits the L2 (kTiledMaxTileBytes).  A workgroup of `threads`
// threads moves one segment of one row, cpt chunks per thread.  False when no shape fits: segments would be
// narrower than 4 KiB, or more than 8.
static bool tiled_shape(const fusco_layout *L, int Ct, int &threads, int &cpt, int &segs, int &per)
{
    int max_chunks = (int)std::min<size_t>(1024, kTiledMaxTileBytes / 16 / (size_t)L->tile_tokens);
    if (max_chunks < 1 || Ct < 1) return false;
    if (Ct > max_chunks) max_chunks = max_chunks / kWave * kWave;   // segments are whole KiB
    if (max_chunks < 1) return false;
    segs = (Ct + max_chunks - 1) / max_chunks;
    per = segs > 1 ? round_up((Ct + segs - 1) / segs, kWave) : Ct;   // segments start on 1 KiB boundaries of the row
    // measured at 8192 tokens x 8: two segments win up to 16 KiB rows (190 against 205 us at 15.5 KiB); from there
    // to 64 KiB rows (five segments) the tiled kernel takes as long as the token walk, and the combine that follows
    // is 5-8 % faster after it, because its stores leave nothing dirty in the memory-side cache
    if (segs > 8 || (segs > 1 && per < 256)) return false;
    cpt = per >= 512 ? 4 : (per >= 128 ? 2 : 1);
    threads = std::min(256, round_up((per + cpt - 1) / cpt, kWave));
    return true;
}

// the conditions under which fusco_dispatch moves the rows tile by tile in transfer order
static bool dispatch_in_transfer_order(const fusco_layout *L, size_t row_bytes, size_t aux_row_bytes, bool expert,
                                       bool wire, bool two_hop)
{
    const int which = g_dispatch_kernel.load(std::memory_order_relaxed);
    if (which == 1) return false;
    int threads, cpt, segs, per;
    if (!(expert && !wire && !two_hop && L->k >= 2 && L->tile_count >= kTiledMinTiles &&
          tiled_shape(L, (int)((row_bytes + aux_row_bytes) / 16), threads, cpt, segs, per)))
        return false;
    if (which == 2) return true;
    // Sizes at which the token walk is as good or better (measured, 8 rows per token):
    // - an expert tensor that fits the memory-side cache: the walk's plain stores leave it there for its reader;
    // - rows shorter than 8 KiB together with a source tensor that would be taken in chunks (more than 128 MiB),
    //   and rows shorter than 4 KiB already with one of 128 MiB, which does not stay in that cache next to the
    //   output of a combine of the same size: the tiles' short runs then lose to the walk;
    // - fewer than 8 rows per token together with a source tensor of more than 128 MiB: a source row is then
    //   fetched for few uses, and the tiles lose to the walk with 4 rows per token (282 against 218 us at 32768
    //   tokens of 7 KiB, 209 against 177 us at 16384 tokens of 12 KiB) and with 5 or 6 rows per token when the rows
    //   are moved in column segments (358 against 303 us at 16384 tokens of 14 KiB, 6 rows per token); whole rows
    //   of 8-10 KiB with 5 or 6 rows per token come out even or up to 2 % ahead in the step.
    const size_t row = row_bytes + aux_row_bytes, source = (size_t)L->N * row;
    const size_t limit = g_source_chunk_bytes.load(std::memory_order_relaxed);
    if ((size_t)L->P * row <= kCacheBytes) return false;
    if (row < kTiledShortRowBytes && source > limit) return false;
    if (row < kTiledShortRowBytes / 2 && source >= limit) return false;
    if (source > limit && !(L->k >= 8 || (L->k >= 5 && segs == 1))) return false;
    return true;
}

int fusco_dispatch_in_transfer_order(const fusco_layout *L, size_t row_bytes, size_t aux_row_bytes, uint32_t flags)
{
    if (!layout_ok(L)) return FUSCO_ERR_INVALID_ARG;
    flags &= ~FUSCO_DISPATCH_STREAMING;
    if (flags == 0) flags = FUSCO_DISPATCH_EXPERT;
    if (flags & ~(FUSCO_DISPATCH_EXPERT | FUSCO_DISPATCH_WIRE | FUSCO_DISPATCH_TWO_HOP)) return FUSCO_ERR_UNSUPPORTED;
    return dispatch_in_transfer_order(L, row_bytes, aux_row_bytes, flags & FUSCO_DISPATCH_EXPERT, flags & FUSCO_DISPATCH_WIRE,
                                      flags & FUSCO_DISPATCH_TWO_HOP) ? 1 : 0;
}

int fusco_dispatch(const fusco_layout *L, const void *d_x, size_t row_bytes, const void *d_x_aux,
                   size_t aux_row_bytes, void *d_expert_buf, void *d_expert_aux, void *d_send_buf,
                   void *d_send_aux, uint32_t flags, void *stream)
{
    if (!layout_ok(L)) return FUSCO_ERR_INVALID_ARG;
    const bool streaming = flags & FUSCO_DISPATCH_STREAMING;
    flags &= ~FUSCO_DISPATCH_STREAMING;
    if (flags == 0) flags = FUSCO_DISPATCH_EXPERT;
    if (flags & ~(FUSCO_DISPATCH_EXPERT | FUSCO_DISPATCH_WIRE | FUSCO_DISPATCH_TWO_HOP)) return FUSCO_ERR_UNSUPPORTED;
    const bool two_hop = flags & FUSCO_DISPATCH_TWO_HOP;
    if (two_hop && streaming) return FUSCO_ERR_UNSUPPORTED;   // the second hop reads the first hop's rows at once
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
    a.slot_token = nullptr; a.tile_slots = nullptr; a.tile_cap = 0; a.tile_tokens = 0; a.N = L->N; a.segs = 1; a.seg_chunks = 0;
    a.k = L->k;
    a.C = (int32_t)(row_bytes / 16);
    a.Ca = (int32_t)(aux_row_bytes / 16);
    a.write_expert = expert && !two_hop; a.write_wire = wire;
    const int Ct = a.C + a.Ca;

    // token walk: as many column segments as workgroups of 256 threads x 4 chunks need, the chunks spread evenly
    int segs = (Ct + 1023) / 1024;
    int per = segs > 1 ? round_up((Ct + segs - 1) / segs, kWave) : Ct;   // segments start on 1 KiB boundaries of the row
    int cpt = per >= 512 ? 4 : (per >= 128 ? 2 : 1);
    int threads = std::min(256, round_up((per + cpt - 1) / cpt, kWave));
    hipStream_t s = (hipStream_t)stream;
    ArmedEvents ev;
    if (two_hop) ev.start = ev.stop = nullptr;   // several kernels: armed events are dropped

    // Expert tensor alone, enough tiles to keep every XCD busy, and a tile's source rows small enough to stay
    // in one XCD's 4 MB L2: the rows are moved tile by tile in transfer order (dispatch_tiled_kernel).
    if (dispatch_in_transfer_order(L, row_bytes, aux_row_bytes, expert, wire, two_hop)) {
        a.slot_token = L->slot_token; a.tile_slots = L->tile_slots;
        a.tile_cap = L->tile_tokens * L->k; a.tile_tokens = L->tile_tokens;
        tiled_shape(L, Ct, threads, cpt, segs, per);
        a.segs = segs; a.seg_chunks = per;
        // a source tensor that cannot stay in the memory-side cache is taken in chunks of whole rounds of tiles
        // whose rows fit half of it, every chunk after a sequential read of its source rows (touch_kernel)
        const size_t source_bytes = (size_t)L->N * (row_bytes + aux_row_bytes);
        const size_t chunk_limit = g_source_chunk_bytes.load(std::memory_order_relaxed);
        size_t chunk_tiles = (size_t)L->tile_count;
        const bool chunked = source_bytes > chunk_limit;
        if (chunked) {
            chunk_tiles = chunk_limit / ((size_t)L->tile_tokens * (row_bytes + aux_row_bytes)) / kXcds * kXcds;
            if (chunk_tiles < (size_t)kXcds) chunk_tiles = kXcds;
        }
        // the largest launch: a workgroup per row and segment of the chunk's tiles (checked before anything is launched)
        if ((uint64_t)((chunk_tiles + kXcds - 1) / kXcds) * (uint64_t)a.tile_cap * (uint64_t)segs * kXcds > 0x7fffffffu)
            return FUSCO_ERR_INVALID_ARG;
        const dim3 tblock((unsigned)threads);
        // A source tensor that is taken in one piece has its rows pulled towards the L2 at the start of every tile;
        // taken in chunks, touch_kernel has just read them and the pull only costs (12 KiB segments at 8192 tokens:
        // 322 us without it, 332 us with it).  The workgroups per compute unit are capped by the row size only while
        // the source tensor and an output of its size stay in the memory-side cache from step to step.  Measured
        // with 14 KiB rows, dispatch alone, 8 / 5 workgroups: 8192 tokens (112 MiB) 164 / 155 us, 8704 tokens
        // (119 MiB) 191 / 188 us, 9216 tokens (126 MiB) 205 / 250 us, 32768 tokens without chunks 793 / 923 us.
        const int occ_knob = g_tiled_occupancy.load(std::memory_order_relaxed);
        const int pull_knob = g_tiled_pull.load(std::memory_order_relaxed);
        const bool pull = pull_knob == 0 ? !chunked : pull_knob == 2;
        const int wgs = occ_knob > 0 ? occ_knob
                        : (source_bytes <= kResidentSourceBytes ? tiled_workgroups_per_cu((size_t)per * 16) : 16);
        const size_t lds = lds_for_occupancy(wgs);
        for (size_t tile0 = 0; tile0 < (size_t)L->tile_count; tile0 += chunk_tiles) {
            const size_t tiles_here = std::min(chunk_tiles, (size_t)L->tile_count - tile0);
            const bool first = tile0 == 0, last = tile0 + tiles_here == (size_t)L->tile_count;
            if (chunked) {
                const size_t t0 = tile0 * (size_t)L->tile_tokens;
                const size_t rows = std::min(tiles_here * (size_t)L->tile_tokens, (size_t)L->N - t0);
                const size_t n = rows * (size_t)a.C, na = rows * (size_t)a.Ca;
                launch_args(touch_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, first ? ev.start : nullptr, (hipEvent_t) nullptr,
                       a.x + t0 * (size_t)a.C, n);
                if (na)
                    launch_args(touch_kernel, dim3((unsigned)((na + 255) / 256)), dim3(256), 0, s, (hipEvent_t) nullptr, (hipEvent_t) nullptr,
                           a.x_aux + t0 * (size_t)a.Ca, na);
            }
            const unsigned tblocks = (unsigned)((tiles_here + kXcds - 1) / kXcds) * (unsigned)a.tile_cap * (unsigned)segs * kXcds;
            hipEvent_t e0 = first && !chunked ? ev.start : nullptr, e1 = last ? ev.stop : nullptr;
            const uint32_t tb = (uint32_t)tile0, th = (uint32_t)tiles_here;
            const dim3 tgrid(tblocks);
#define FUSCO_TILED(CPT)                                                                              \
    do {                                                                                              \
        if (a.Ca && pull) launch_args(dispatch_tiled_kernel<CPT, true, true>, tgrid, tblock, lds, s, e0, e1, a, tb, th);        \
        else if (a.Ca) launch_args(dispatch_tiled_kernel<CPT, true, false>, tgrid, tblock, lds, s, e0, e1, a, tb, th);          \
        else if (pull) launch_args(dispatch_tiled_kernel<CPT, false, true>, tgrid, tblock, lds, s, e0, e1, a, tb, th);          \
        else launch_args(dispatch_tiled_kernel<CPT, false, false>, tgrid, tblock, lds, s, e0, e1, a, tb, th);                   \
    } while (0)
            switch (cpt) {
            case 1: FUSCO_TILED(1); break;
            case 2: FUSCO_TILED(2); break;
            default: FUSCO_TILED(4); break;
            }
#undef FUSCO_TILED
        }
        return launch_status();
    }
    if ((uint64_t)L->N * (uint64_t)segs > 0x7fffffffu) return FUSCO_ERR_INVALID_ARG;
    a.segs = segs; a.seg_chunks = per;
    const dim3 grid((unsigned)L->N * (unsigned)segs), block((unsigned)threads);
    {
        // Loads and stores of the walk (dispatch_kernel's MODE).  Tensors of more than 256 MB in all cannot stay in
        // the memory-side cache for their reader, and what plain stores leave of them there dirty only slows the
        // next reader of memory down: they are written with non-temporal stores, as with FUSCO_DISPATCH_STREAMING.
        // Measured in a dispatch + combine loop whose combine reads another tensor, plain / streaming, % of peak:
        // 8192 tokens x 8 rows of 14 KiB 67.0 / 74.8, 16384 x 8 x 4 KiB 66.7 / 76.3, 32768 x 2 x 8 KiB 75.0 / 81.9,
        // 32768 x 4 x 14 KiB 68.6 / 70.5, 65536 x 1 x 8 KiB 73.5 / 75.4; with the combine reading the rows just
        // written 73.7 / 74.6, 71.1 / 76.2, 76.8 / 77.8, 70.0 / 70.3, 73.4 / 74.8.
        const size_t row = row_bytes + aux_row_bytes;
        const size_t written = ((expert && !two_hop ? (size_t)L->P : 0) + (wire ? (size_t)L->send_cap : 0)) * row;
        const bool stream_stores = streaming || (!two_hop && written > kCacheBytes);   // the second hop reads the rows at once
        const bool cached_loads = stream_stores && (size_t)L->N * row <= g_source_chunk_bytes.load(std::memory_order_relaxed);
        const int knob = g_walk_mode.load(std::memory_order_relaxed);
        const int mode = knob > 0 ? knob - 1 : (stream_stores ? 2 : 0) + (cached_loads ? 1 : 0);
#define FUSCO_WALK(CPT)                                                                       \
    switch (mode) {                                                                           \
    case 0: launch(dispatch_kernel<CPT, 0>, grid, block, s, a, ev.start, ev.stop); break;     \
    case 1: launch(dispatch_kernel<CPT, 1>, grid, block, s, a, ev.start, ev.stop); break;     \
    case 2: launch(dispatch_kernel<CPT, 2>, grid, block, s, a, ev.start, ev.stop); break;     \
    default: launch(dispatch_kernel<CPT, 3>, grid, block, s, a, ev.start, ev.stop); break;    \
    }
        switch (cpt) {
        case 1: FUSCO_WALK(1); break;
        case 2: FUSCO_WALK(2); break;
        default: FUSCO_WALK(4); break;
        }
#undef FUSCO_WALK
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
    const int rc = combine_check(d_y, y_dtype, d_w, d_out, out_dtype, H, L->N == 0, (int64_t)L->N);
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
    const int rc = combine_check(d_y, y_dtype, d_w, d_out, out_dtype, H, L->N == 0, (int64_t)L->send_cap);
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
    a.first = 0;
    a.n_rows = L->send_cap;
    int threads;
    combine_shape(a.C, threads, a.segs);
    const dim3 grid((unsigned)L->send_cap * (unsigned)a.segs);
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
    if (!layout_ok(L) || !layout_ok(Lr) || (!d_topk_idx && L->N > 0) || (!d_topk_dev && L->N > 0) || !d_scratch)
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
    const int rc = combine_check(d_y, y_dtype, d_w, d_out, out_dtype, H, L->N == 0, (int64_t)L->N);
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

int fusco_cross_node_load(const fusco_layout *L, int32_t devices_per_node, int32_t home_node, size_t row_bytes,
                          int64_t *d_load, void *stream)
{
    if (!layout_ok(L) || !d_load || ((uintptr_t)d_load & 7u)) return FUSCO_ERR_INVALID_ARG;
    if (devices_per_node < 1 || L->D % devices_per_node != 0) return FUSCO_ERR_INVALID_ARG;
    if (home_node < 0 || home_node >= L->D / devices_per_node) return FUSCO_ERR_INVALID_ARG;
    if (row_bytes == 0 || row_bytes > FUSCO_MAX_ROW_BYTES) return FUSCO_ERR_INVALID_ARG;
    hipLaunchKernelGGL(cross_node_load_kernel, dim3(1), dim3(kWave), 0, (hipStream_t)stream, L->send_count, L->D,
                       devices_per_node, home_node, (uint64_t)row_bytes, d_load);
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

int fusco_probe_pieces(void *d_buf, size_t bytes, int write, uint32_t run_pieces, int scatter, uint32_t *d_sink,
                       void *stream)
{
    if (!d_buf || !aligned16(d_buf) || bytes == 0 || bytes % 4096 != 0 || bytes / 4096 > 0x7FFFFFFFu)
        return FUSCO_ERR_INVALID_ARG;
    const uint32_t pieces = (uint32_t)(bytes / 4096);
    if (scatter ? pieces < 3 : (run_pieces == 0 || pieces % 8u != 0 || (pieces / 8u) % run_pieces != 0))
        return FUSCO_ERR_INVALID_ARG;
    if (!write && !d_sink) return FUSCO_ERR_INVALID_ARG;
    ProbePiecesArgs a;
    a.buf = (u32x4 *)d_buf; a.sink = d_sink; a.pieces = pieces;
    a.run = scatter ? 1u : run_pieces;
    a.mul = scatter ? coprime_near(pieces, 0.6180339887498949) : 0u;
    hipStream_t s = (hipStream_t)stream;
    if (write) hipLaunchKernelGGL(probe_pieces_kernel<true>, dim3(pieces), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(probe_pieces_kernel<false>, dim3(pieces), dim3(256), 0, s, a);
    return launch_status();
}

int fusco_probe_consume_slices(const void *d_stream, uint64_t total_bytes, uint64_t slice_bytes,
                               const uint32_t *d_slice_fill, uint32_t max_polls, uint32_t *d_report, void *stream)
{
    if (!d_stream || !aligned16(d_stream) || !d_slice_fill || !d_report) return FUSCO_ERR_INVALID_ARG;
    if (slice_bytes == 0 || slice_bytes % 16 != 0 || slice_bytes > ((uint64_t)1 << 31) || total_bytes % 16 != 0)
        return FUSCO_ERR_INVALID_ARG;
    const uint64_t slices = (total_bytes + slice_bytes - 1) / slice_bytes;
    if (slices > (1u << 20) || max_polls > (1u << 24)) return FUSCO_ERR_INVALID_ARG;
    if (slices == 0) return FUSCO_OK;
    ConsumeArgs a;
    a.stream = (const u32x4 *)d_stream; a.slice_fill = d_slice_fill; a.total = total_bytes; a.slice_bytes = slice_bytes;
    a.n_slices = (uint32_t)slices; a.max_polls = max_polls; a.report = d_report;
    hipLaunchKernelGGL(consume_slices_kernel, dim3(1), dim3(256), 0, (hipStream_t)stream, a);
    return launch_status();
}

int fusco_probe_dispatch_kernel(int which)
{
    if (which > 2) return FUSCO_ERR_INVALID_ARG;
    return which < 0 ? g_dispatch_kernel.load() : g_dispatch_kernel.exchange(which);
}

int fusco_probe_dispatch_walk(int which)
{
    if (which > 4) return FUSCO_ERR_INVALID_ARG;
    return which < 0 ? g_walk_mode.load() : g_walk_mode.exchange(which);
}

int fusco_probe_dispatch_pull(int which)
{
    if (which > 2) return FUSCO_ERR_INVALID_ARG;
    return which < 0 ? g_tiled_pull.load() : g_tiled_pull.exchange(which);
}

int fusco_probe_dispatch_occupancy(int wgs)
{
    if (wgs > 16 || (wgs > 0 && wgs < 3)) return FUSCO_ERR_INVALID_ARG;   // 16: no cap
    return wgs < 0 ? g_tiled_occupancy.load() : g_tiled_occupancy.exchange(wgs);
}

size_t fusco_probe_source_chunk_bytes(size_t bytes)
{
    return bytes ? g_source_chunk_bytes.exchange(bytes) : g_source_chunk_bytes.load();
}

int fusco_probe_time_next_call(void *start_event, void *stop_event)
{
    if (!start_event || !stop_event) return FUSCO_ERR_INVALID_ARG;
    g_time_start = (hipEvent_t)start_event;
    g_time_stop = (hipEvent_t)stop_event;
    return FUSCO_OK;
}

}   // extern "C"
