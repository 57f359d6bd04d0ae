// Host side: argument checks shared by the entry points, kernel launch helpers, per-call timing events.
#ifndef FUSCO_CSRC_LAUNCH_H
#define FUSCO_CSRC_LAUNCH_H

#include "common.h"
#include "planner.h"
#include "movers.h"
#include "segments.h"
#include "probes.h"

namespace {

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

// the same for kernels with several arguments; `lds` bytes of dynamic LDS (which the kernels do not use: asking
// for it caps the number of workgroups a compute unit holds at once)
template <typename K, typename... A>
void launch_args(K kernel, dim3 grid, dim3 block, size_t lds, hipStream_t s, hipEvent_t e0, hipEvent_t e1, A... args)
{
    if (e0 || e1) hipExtLaunchKernelGGL(kernel, grid, block, (unsigned)lds, s, e0, e1, 0, args...);
    else hipLaunchKernelGGL(kernel, grid, block, (unsigned)lds, s, args...);
}

// Workgroup shape of combine_kernel for rows of C chunks: as many column segments as 1024 threads need, the
// threads spread evenly over them (1280 chunks: two workgroups of 640 threads, not 1024 + 256).
inline void combine_shape(int C, int &threads, int &segs)
{
    segs = (C + 1023) / 1024;
    if (segs < 1) segs = 1;
    threads = round_up((C + segs - 1) / segs, kWave);
}

// Rows that a thread of combine_kernel has in flight at a time (JU).  Inputs that are bound by memory run a few
// percent faster with two than with all eight of a token's rows (8192 tokens x 8 rows of 14 KiB: 172 us against
// 178 us; 4096 tokens: 88 against 92 us; 32768 x 8 x 2 KiB: 95 against 97 us; 8 KiB rows: the same); small inputs
// are bound by latency and take the token's rows at once.
constexpr size_t kCombineLatencyBoundBytes = (size_t)64 << 20;

template <bool Y_BF16, bool OUT_BF16>
void launch_combine(CombineArgs a, int N, hipStream_t s, hipEvent_t e0, hipEvent_t e1)
{
    int threads;
    combine_shape(a.C, threads, a.segs);
    a.n_rows = N;
    const dim3 grid((unsigned)N * (unsigned)a.segs), block((unsigned)threads);
    if ((size_t)N * (size_t)a.k * (size_t)a.C * 16 < kCombineLatencyBoundBytes)
        launch(combine_kernel<Y_BF16, OUT_BF16, 1, 8>, grid, block, s, a, e0, e1);
    else
        launch(combine_kernel<Y_BF16, OUT_BF16, 1, 2>, grid, block, s, a, e0, e1);
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
// walk_rows: rows the combine walks over (tokens, or send rows); the launch needs a workgroup per row and column segment
int combine_check(const void *d_y, int y_dtype, const float *d_w, const void *d_out, int out_dtype, int32_t H,
                  bool empty, int64_t walk_rows)
{
    if (H <= 0 || (!empty && (!d_y || !d_w || !d_out))) return FUSCO_ERR_INVALID_ARG;
    if ((y_dtype != FUSCO_BF16 && y_dtype != FUSCO_F32) || (out_dtype != FUSCO_BF16 && out_dtype != FUSCO_F32))
        return FUSCO_ERR_UNSUPPORTED;
    const size_t y_row = (size_t)H * (y_dtype == FUSCO_BF16 ? 2 : 4);
    if (y_row % 16 != 0 || y_row / 16 > kMaxRowChunks) return FUSCO_ERR_INVALID_ARG;
    if (!aligned16(d_y) || !aligned16(d_out) || ((uintptr_t)d_w & 3u)) return FUSCO_ERR_INVALID_ARG;
    int threads, segs;
    combine_shape((int)(y_row / 16), threads, segs);
    if (walk_rows * segs > 0x7fffffff) return FUSCO_ERR_INVALID_ARG;
    return FUSCO_OK;
}

// Where the combine walk starts.  Right after a dispatch of the same tokens the memory-side cache (256 MB)
// still holds the rows written for the last tokens.  Measured on MI355X (8192 tokens x 8 rows of 14 KiB): a
// walk that starts about 110-220 MiB of rows before the end, goes up to the last token and then wraps to
// token 0 is 7 us (2 %) faster than a walk from the last token down, and 25 us faster than one from token 0
// up.  That holds after a dispatch that writes with plain stores (the token walk); the tiled dispatch's
// streaming stores leave nothing in that cache, and when y comes from somewhere else the order makes no
// difference either.
constexpr size_t kRecentRowBytes = (size_t)160 << 20;

int combine_first_row(int N, int k, size_t row_bytes)
{
    const size_t per_token = (size_t)k * row_bytes;
    const size_t recent = kRecentRowBytes / (per_token ? per_token : 1);
    return recent >= (size_t)N ? 0 : N - (int)recent;
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
    a.first = combine_first_row(N, k, (size_t)a.C * 16);
    if (y_dtype == FUSCO_BF16 && out_dtype == FUSCO_BF16) launch_combine<true, true>(a, N, s, e0, e1);
    else if (y_dtype == FUSCO_BF16) launch_combine<true, false>(a, N, s, e0, e1);
    else if (out_dtype == FUSCO_BF16) launch_combine<false, true>(a, N, s, e0, e1);
    else launch_combine<false, false>(a, N, s, e0, e1);
}

}   // namespace

#endif
