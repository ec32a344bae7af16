// Wave / block prefix sums used by the compaction passes (active sets, boundary sampling).
#pragma once
#include "common.h"

namespace gnnhot {

__device__ __forceinline__ int wave_inclusive_scan(int x) {
    const int lane = lane_id();
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        int y = __shfl_up(x, d, kWave);
        if (lane >= d) x += y;
    }
    return x;
}

// Exclusive prefix of x over a block of NT threads (NT a multiple of 64, <= 1024).
// s_part must hold NT/64 ints.  *total receives the block sum.  Contains two barriers.
template <int NT>
__device__ __forceinline__ int block_exclusive_scan(int x, int* s_part, int* total) {
    constexpr int NW = NT / kWave;
    const int inc = wave_inclusive_scan(x);
    const int w = (int)(threadIdx.x >> 6);
    if (lane_id() == kWave - 1) s_part[w] = inc;
    __syncthreads();
    int base = 0, sum = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        int p = s_part[i];
        if (i < w) base += p;
        sum += p;
    }
    *total = sum;
    __syncthreads();
    return base + inc - x;
}

// In-place exclusive scan of counts[0..n) by ONE block of 1024 threads (n up to a few
// million: each thread walks a contiguous chunk).  counts[n] receives the total.
__device__ __forceinline__ int64_t single_block_exclusive_scan(int32_t* counts, int64_t n, int* s_part) {
    const int64_t chunk = (n + 1023) / 1024;
    const int64_t lo = (int64_t)threadIdx.x * chunk;
    const int64_t hi = lo + chunk < n ? lo + chunk : n;
    int local = 0;
    for (int64_t i = lo; i < hi; ++i) local += counts[i];
    int total;
    int run = block_exclusive_scan<1024>(local, s_part, &total);
    for (int64_t i = lo; i < hi; ++i) {
        int c = counts[i];
        counts[i] = run;
        run += c;
    }
    if (threadIdx.x == 0) counts[n] = total;
    return (int64_t)total;
}

// ---- counts[0..n) -> offsets[0..n] (exclusive prefix, offsets[n] = total), n up to 2^31 --------------------
// Three launches: per-block sums (1024 counts per block), one block scans the sums, every block rescans its own
// counts on top of its base.  `sums` is scratch of offsets_scan_blocks(n) + 1 ints.  The kernels are static: every
// translation unit that includes this header gets its own copy.
constexpr int kScanBlock = 1024;  // counts per block (256 threads x 4)

inline int32_t offsets_scan_blocks(int32_t n) { return n > 0 ? (n + kScanBlock - 1) / kScanBlock : 1; }

static __global__ __launch_bounds__(256) void scan_block_sums_kernel(const int32_t* __restrict__ counts, int32_t n,
                                                                      int32_t* __restrict__ sums) {
    __shared__ int s_part[4];
    const int64_t base = (int64_t)blockIdx.x * kScanBlock + threadIdx.x * 4;
    int c = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k)
        if (base + k < n) c += counts[base + k];
    int total;
    block_exclusive_scan<256>(c, s_part, &total);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

static __global__ __launch_bounds__(1024) void scan_sums_kernel(int32_t* __restrict__ sums, int32_t n_blocks,
                                                                 int64_t* __restrict__ out_total) {
    __shared__ int s_part[16];
    const int64_t total = single_block_exclusive_scan(sums, n_blocks, s_part);
    if (threadIdx.x == 0) *out_total = total;
}

static __global__ __launch_bounds__(256) void scan_offsets_kernel(const int32_t* __restrict__ counts, int32_t n,
                                                                   const int32_t* __restrict__ sums, int32_t n_blocks,
                                                                   int32_t* __restrict__ offsets) {
    __shared__ int s_part[4];
    const int64_t base = (int64_t)blockIdx.x * kScanBlock + threadIdx.x * 4;
    int c[4], tot = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        c[k] = base + k < n ? counts[base + k] : 0;
        tot += c[k];
    }
    int total;
    int run = block_exclusive_scan<256>(tot, s_part, &total) + sums[blockIdx.x];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        if (base + k < n) offsets[base + k] = run;
        run += c[k];
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) offsets[n] = sums[n_blocks];
}

// Enqueues the three launches.  With n == 0: offsets[0] = 0 and *out_total = 0.
inline int32_t counts_to_offsets(const int32_t* counts, int32_t n, int32_t* sums, int32_t* offsets, int64_t* out_total,
                                 hipStream_t stream) {
    const int32_t n_blocks = offsets_scan_blocks(n);
    if (n > 0) {
        scan_block_sums_kernel<<<n_blocks, 256, 0, stream>>>(counts, n, sums);
        GNN_LAUNCH_CHECK("scan_block_sums_kernel");
    }
    scan_sums_kernel<<<1, 1024, 0, stream>>>(sums, n > 0 ? n_blocks : 0, out_total);
    GNN_LAUNCH_CHECK("scan_sums_kernel");
    scan_offsets_kernel<<<n_blocks, 256, 0, stream>>>(counts, n, sums, n > 0 ? n_blocks : 0, offsets);
    GNN_LAUNCH_CHECK("scan_offsets_kernel");
    return GNN_OK;
}

}  // namespace gnnhot
