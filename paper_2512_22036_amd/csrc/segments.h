// Segment-descriptor engine kernels: variable-size segments described by (offset, size) lists.
#ifndef FUSCO_CSRC_SEGMENTS_H
#define FUSCO_CSRC_SEGMENTS_H

#include "common.h"
#include "movers.h"

namespace {

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
        // in range without any sum that could wrap: a unit fits iff its start is at most bytes - 16, and a
        // start below `intra` means offset + intra wrapped around 2^64 (e.g. a negative offset)
        const bool src_in = a.src_bytes >= 16 && so <= a.src_bytes - 16 && so >= intra;
        const bool dst_in = a.dst_bytes >= 16 && dofs <= a.dst_bytes - 16 && dofs >= intra;
        if (((so | dofs) & 15u) || !src_in || !dst_in) {
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
        if constexpr (SLICES) store16_system((u32x4 *)(a.dst + dst_at[r]), v[r]);
        else *(u32x4 *)(a.dst + dst_at[r]) = v[r];
    }
    if (skipped) atomicAdd(a.status, skipped);
    if constexpr (SLICES) {
        // A slice counts bytes only once they are in memory: the stores above are write-through at
        // system scope (sc0 sc1), every thread waits for its own to complete, and only then one thread
        // adds the bytes the workgroup has really written (skipped units are left out, so a slice with
        // holes never reaches its size) with a system-scope atomic.  (A device-wide release fence
        // would do too, but it writes back the whole L2 of the XCD each time.)
        __shared__ int skipped_total;
        if (threadIdx.x == 0) skipped_total = 0;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (skipped) atomicAdd(&skipped_total, skipped);
        __syncthreads();
        if (threadIdx.x == 0) {
            const uint64_t left = total - base;
            const uint32_t mine = (uint32_t)(left < kSegBlockBytes ? left : kSegBlockBytes);
            __hip_atomic_fetch_add(a.slice_fill + base / a.slice_bytes, mine - 16u * (uint32_t)skipped_total,
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
}

}   // namespace

#endif
