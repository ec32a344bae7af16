// Ordering keys of the sampling kernels: the seeded counter-based edge hash of the boundary sampler (paper section
// 5.3; splitmix64's output function) and lexicographic (key, id) comparison.
#pragma once
#include "common.h"

namespace gnnhot {

// splitmix64 output function: golden-ratio increment, two xor-shift-multiply rounds, xor-shift.
__host__ __device__ __forceinline__ uint64_t mix64(uint64_t x) {
    x += 0x9E3779B97F4A7C15ull;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}

__device__ __forceinline__ uint64_t edge_key(uint64_t seed_hop_mixed, uint64_t v, uint64_t u) {
    return mix64(mix64(seed_hop_mixed ^ v) ^ u);
}

__device__ __forceinline__ bool in_set(const uint32_t* __restrict__ bitmap, int32_t u) {
    return (bitmap[u >> 5] >> (u & 31)) & 1u;
}

// (key, id) pairs ordered lexicographically
__device__ __forceinline__ bool pair_less(uint64_t ka, int32_t ua, uint64_t kb, int32_t ub) {
    return ka < kb || (ka == kb && ua < ub);
}

}  // namespace gnnhot
