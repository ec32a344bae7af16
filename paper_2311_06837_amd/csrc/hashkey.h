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

// ---- a wavefront's list of (key, id) pairs in LDS: the selection step shared by the traversal and the layer masks ----

// The k-th smallest of the n (> k >= 1) distinct pairs of the list: k rounds of "smallest pair above the previous
// one".  Every lane returns the same pair.
__device__ __forceinline__ void wave_list_kth(const uint64_t* key, const int32_t* id, int32_t n, int32_t k, int lane, uint64_t& thr_k,
                                              int32_t& thr_u) {
    uint64_t prev_k = 0ull;
    int32_t prev_u = -1;
    for (int32_t round = 0; round < k; ++round) {
        uint64_t best_k = ~0ull;
        int32_t best_u = 0x7fffffff;
        for (int32_t j = lane; j < n; j += kWave) {
            const uint64_t kj = key[j];
            const int32_t uj = id[j];
            if (pair_less(prev_k, prev_u, kj, uj) && pair_less(kj, uj, best_k, best_u)) {
                best_k = kj;
                best_u = uj;
            }
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            const uint64_t ok = __shfl_xor(best_k, d, kWave);
            const int32_t ou = __shfl_xor(best_u, d, kWave);
            if (pair_less(ok, ou, best_k, best_u)) {
                best_k = ok;
                best_u = ou;
            }
        }
        prev_k = best_k;
        prev_u = best_u;
    }
    thr_k = prev_k;
    thr_u = prev_u;
}

// Drops the pairs above (thr_k, thr_u) from the list, in place and in order; returns how many are left.
__device__ __forceinline__ int32_t wave_list_keep_below(uint64_t* key, int32_t* id, int32_t n, uint64_t thr_k, int32_t thr_u, int lane) {
    const uint64_t lanes_below = (1ull << lane) - 1ull;
    int32_t out = 0;
    for (int32_t base = 0; base < n; base += kWave) {   // front to back: targets lie at or before the chunk being read
        const int32_t j = base + lane;
        const uint64_t kj = j < n ? key[j] : 0ull;
        const int32_t uj = j < n ? id[j] : 0;
        const bool keep = j < n && !pair_less(thr_k, thr_u, kj, uj);
        const uint64_t km = __ballot(keep);
        wave_lds_sync();   // the chunk has been read by every lane
        if (keep) {
            const int32_t pos = out + __popcll(km & lanes_below);
            key[pos] = kj;
            id[pos] = uj;
        }
        out += __popcll(km);
        wave_lds_sync();
    }
    return out;
}

}  // namespace gnnhot
