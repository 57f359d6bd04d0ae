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

}   // namespace

#endif
