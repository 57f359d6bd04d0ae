// Measurement-aid kernels: plain copy and row traffic of a chosen shape.
#ifndef FUSCO_CSRC_PROBES_H
#define FUSCO_CSRC_PROBES_H

#include "common.h"
#include "movers.h"

namespace {

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

// Measurement aid: a buffer as a stream of 4 KiB pieces, one 16-byte access per thread, with a chosen
// assignment of pieces to XCDs.  Workgroups are handed to the 8 XCDs in turn (workgroup b runs on XCD
// b mod 8), so workgroup b = 8 i + x takes piece ((i / run) * 8 + x) * run + i mod run: every XCD works
// through runs of `run` consecutive pieces, and the 8 runs of a round are neighbours in memory.  run == 1
// walks the buffer in launch order.  With mul != 0 piece b * mul mod pieces is taken instead (scattered).
struct ProbePiecesArgs {
    u32x4 *buf;
    uint32_t *sink;
    uint32_t pieces, run, mul;
};

template <bool WRITE>
__global__ __launch_bounds__(256) void probe_pieces_kernel(ProbePiecesArgs a)
{
    const uint32_t b = blockIdx.x;
    uint32_t p;
    if (a.mul) {
        p = (uint32_t)((uint64_t)b * a.mul % a.pieces);
    } else {
        const uint32_t x = b & 7u, i = b >> 3, g = i / a.run;
        p = (g * 8u + x) * a.run + (i - g * a.run);
    }
    u32x4 *at = a.buf + (size_t)p * 256 + threadIdx.x;
    if constexpr (WRITE) {
        const u32x4 v = {p, threadIdx.x, b, 0x50494543u};
        *at = v;
    } else {
        const u32x4 v = load16_stream(at);
        if ((v.x ^ v.y ^ v.z ^ v.w) == 0x9E3779B9u && a.sink) a.sink[0] = p;
    }
}

// Validation aid for the slice protocol of the segment engine: the consumer side.  One workgroup walks
// the slices of a packed stream in order; for each it polls the slice's byte counter (acquire loads at
// system scope, a bounded number of polls over the whole walk) and, once the counter has reached the
// slice's size, adds up the slice's 32-bit words.  It always terminates: when the poll budget is used
// up the remaining slices are reported as not ready.
// report[4 s .. 4 s + 3] = { 1 if slice s was seen complete else 0, polls spent waiting for it,
//                            low and high half of the 64-bit sum of its 32-bit words }.
struct ConsumeArgs {
    const u32x4 *stream;
    const uint32_t *slice_fill;
    uint64_t total, slice_bytes;
    uint32_t n_slices, max_polls;
    uint32_t *report;
};

__global__ __launch_bounds__(256) void consume_slices_kernel(ConsumeArgs a)
{
    __shared__ unsigned long long sum;
    __shared__ uint32_t ready, polls_here;
    uint32_t budget = a.max_polls;   // kept in step by every thread through the shared polls_here
    for (uint32_t s = 0; s < a.n_slices; ++s) {
        const uint64_t begin = (uint64_t)s * a.slice_bytes;
        const uint64_t left = a.total - begin;
        const uint32_t expect = (uint32_t)(left < a.slice_bytes ? left : a.slice_bytes);
        if (threadIdx.x == 0) {
            uint32_t polls = 0, seen;
            for (;;) {
                seen = __hip_atomic_load(a.slice_fill + s, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_SYSTEM);
                if (seen >= expect || polls >= budget) break;
                ++polls;
                __builtin_amdgcn_s_sleep(8);
            }
            ready = seen >= expect ? 1u : 0u;
            polls_here = polls;
            sum = 0;
        }
        __syncthreads();
        budget -= polls_here;
        if (ready) {
            // every thread orders its own reads of the slice after the counter
            (void)__hip_atomic_load(a.slice_fill + s, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_SYSTEM);
            unsigned long long mine = 0;
            const u32x4 *p = a.stream + begin / 16;
            for (uint32_t u = threadIdx.x; u < expect / 16; u += 256) {
                const u32x4 v = p[u];
                mine += (unsigned long long)v.x + v.y + v.z + v.w;
            }
            atomicAdd(&sum, mine);
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            a.report[4 * s + 0] = ready;
            a.report[4 * s + 1] = polls_here;
            a.report[4 * s + 2] = (uint32_t)sum;
            a.report[4 * s + 3] = (uint32_t)(sum >> 32);
        }
        __syncthreads();
    }
}

}   // namespace

#endif