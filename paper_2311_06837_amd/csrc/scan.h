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

}  // namespace gnnhot
