// Expansion-aware sampling, boundary only (paper section 5.3): dependencies between inner
// (target) vertices stay whole; of the neighbours that lie outside the target set each
// target keeps at most `fanout`.  The choice is a seeded counter-based hash of the edge
// (no generator state, no dependence on thread order): the `fanout` smallest (key, id) win.
//
// One wavefront per target row.  Count pass: ballots over the row give |row in T| and the
// number of outside neighbours; a three-kernel scan turns counts into row offsets.  Fill
// pass: when a row has more than `fanout` outside neighbours the wave finds the fanout-th
// smallest (key, id) by `fanout` rounds of "smallest pair above the previous one" (the row
// is re-read from cache each round), then emits the row in its original ascending order
// through a ballot-prefix compaction.  Bound: HBM (one streaming read of the target rows).
#include "common.h"
#include "scan.h"

namespace gnnhot {

// splitmix64 output function: golden-ratio increment, two xor-shift-multiply rounds, xor-shift.
__device__ __forceinline__ uint64_t mix64(uint64_t x) {
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

__global__ __launch_bounds__(256) void sb_count_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                                                       int32_t n, const uint32_t* __restrict__ tbits,
                                                       const int32_t* __restrict__ targets, int32_t n_targets, int32_t fanout,
                                                       int32_t* __restrict__ counts) {
    const int lane = lane_id();
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    if (i >= n_targets) return;
    const int32_t v = targets[i];
    int32_t n_in = 0, n_ext = 0;
    if (v >= 0 && v < n) {
        const int32_t s = row_ptr[v], e = row_ptr[v + 1];
        for (int32_t base = s; base < e; base += kWave) {
            const int32_t p = base + lane;
            const bool valid = p < e;
            const bool inner = valid && in_set(tbits, col_idx[p]);
            n_in += __popcll(__ballot(inner));
            n_ext += __popcll(__ballot(valid && !inner));
        }
    }
    if (lane == 0) counts[i] = n_in + (n_ext < fanout ? n_ext : fanout);
}

constexpr int kScanBlock = 1024;  // counts per block in the offset scan (256 threads x 4)

__global__ __launch_bounds__(256) void sb_block_sums_kernel(const int32_t* __restrict__ counts, int32_t n, int32_t* __restrict__ sums) {
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

__global__ __launch_bounds__(1024) void sb_scan_sums_kernel(int32_t* __restrict__ sums, int32_t n_blocks, int64_t* __restrict__ out_nnz) {
    __shared__ int s_part[16];
    const int64_t total = single_block_exclusive_scan(sums, n_blocks, s_part);
    if (threadIdx.x == 0) *out_nnz = total;
}

__global__ __launch_bounds__(256) void sb_offsets_kernel(const int32_t* __restrict__ counts, int32_t n, const int32_t* __restrict__ sums,
                                                         int32_t n_blocks, int32_t* __restrict__ out_row_ptr) {
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
        if (base + k < n) out_row_ptr[base + k] = run;
        run += c[k];
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) out_row_ptr[n] = sums[n_blocks];
}

__global__ __launch_bounds__(256) void sb_fill_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                                                      int32_t n, const uint32_t* __restrict__ tbits,
                                                      const int32_t* __restrict__ targets, int32_t n_targets, int32_t fanout,
                                                      uint64_t seed_hop_mixed, const int32_t* __restrict__ out_row_ptr,
                                                      int32_t* __restrict__ out_col_idx, int64_t capacity) {
    const int lane = lane_id();
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    if (i >= n_targets) return;
    const int32_t v = targets[i];
    if (v < 0 || v >= n) return;
    const int32_t s = row_ptr[v], e = row_ptr[v + 1];

    int32_t n_ext = 0;
    for (int32_t base = s; base < e; base += kWave) {
        const int32_t p = base + lane;
        n_ext += __popcll(__ballot(p < e && !in_set(tbits, col_idx[p])));
    }
    // threshold pair: outside neighbours with (key, id) <= (thr_k, thr_u) are kept
    uint64_t thr_k = ~0ull;
    int32_t thr_u = 0x7fffffff;
    if (fanout == 0) {
        thr_k = 0ull;
        thr_u = -1;  // nothing is <= (0, -1): ids are non-negative
    } else if (n_ext > fanout) {
        uint64_t prev_k = 0ull;
        int32_t prev_u = -1;
        for (int32_t round = 0; round < fanout; ++round) {
            uint64_t best_k = ~0ull;
            int32_t best_u = 0x7fffffff;
            for (int32_t p = s + lane; p < e; p += kWave) {
                const int32_t u = col_idx[p];
                if (in_set(tbits, u)) continue;
                const uint64_t k = edge_key(seed_hop_mixed, (uint64_t)v, (uint64_t)u);
                if (pair_less(prev_k, prev_u, k, u) && pair_less(k, u, best_k, best_u)) {
                    best_k = k;
                    best_u = u;
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

    int64_t pos = out_row_ptr[i];
    for (int32_t base = s; base < e; base += kWave) {
        const int32_t p = base + lane;
        bool keep = false;
        int32_t u = 0;
        if (p < e) {
            u = col_idx[p];
            if (in_set(tbits, u)) {
                keep = true;
            } else {
                const uint64_t k = edge_key(seed_hop_mixed, (uint64_t)v, (uint64_t)u);
                keep = !pair_less(thr_k, thr_u, k, u);
            }
        }
        const uint64_t m = __ballot(keep);
        const int64_t my = pos + __popcll(m & ((1ull << lane) - 1ull));
        if (keep && my < capacity) out_col_idx[my] = u;
        pos += __popcll(m);
    }
}

}  // namespace gnnhot

using namespace gnnhot;

extern "C" int32_t gnn_sample_boundary(const gnn_csr* g, const uint32_t* target_bitmap, const int32_t* targets, int32_t n_targets,
                                       int32_t fanout, int32_t hops, uint64_t seed, int32_t* out_row_ptr, int32_t* out_col_idx,
                                       int64_t out_capacity, int64_t* out_nnz, int64_t* out_nnz_host, void* ws, size_t* ws_bytes,
                                       void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    GNN_CHECK(check_csr(g, "g"));
    GNN_REQUIRE(fanout >= 0, GNN_ERR_INVALID_ARG, "fanout < 0");
    GNN_REQUIRE(hops == 1, GNN_ERR_UNSUPPORTED, "only hops = 1 is implemented (got %d)", hops);
    GNN_REQUIRE(n_targets >= 0, GNN_ERR_INVALID_ARG, "n_targets < 0");
    const int32_t n_blocks = n_targets > 0 ? (n_targets + kScanBlock - 1) / kScanBlock : 1;
    WsCarver carve(ws);
    int32_t* counts = carve.take<int32_t>((size_t)n_targets + 1);
    int32_t* sums = carve.take<int32_t>((size_t)n_blocks + 1);
    bool query;
    GNN_CHECK(ws_protocol(ws, ws_bytes, carve.used, &query));
    if (query) return GNN_OK;
    GNN_REQUIRE(out_row_ptr != nullptr, GNN_ERR_INVALID_ARG, "out_row_ptr is NULL");
    GNN_REQUIRE(n_targets == 0 || (targets != nullptr && target_bitmap != nullptr), GNN_ERR_INVALID_ARG, "targets / bitmap is NULL");
    const int wave_grid = grid_for((int64_t)n_targets * kWave, 256, 1 << 30);

    if (out_col_idx == nullptr) {  // count pass
        GNN_REQUIRE(out_nnz != nullptr, GNN_ERR_INVALID_ARG, "out_nnz is NULL");
        if (n_targets > 0) {
            sb_count_kernel<<<wave_grid, 256, 0, stream>>>(g->row_ptr, g->col_idx, g->n_rows, target_bitmap, targets, n_targets, fanout,
                                                           counts);
            GNN_LAUNCH_CHECK("sb_count_kernel");
            sb_block_sums_kernel<<<n_blocks, 256, 0, stream>>>(counts, n_targets, sums);
            GNN_LAUNCH_CHECK("sb_block_sums_kernel");
        }
        sb_scan_sums_kernel<<<1, 1024, 0, stream>>>(sums, n_targets > 0 ? n_blocks : 0, out_nnz);
        GNN_LAUNCH_CHECK("sb_scan_sums_kernel");
        sb_offsets_kernel<<<n_blocks, 256, 0, stream>>>(counts, n_targets, sums, n_targets > 0 ? n_blocks : 0, out_row_ptr);
        GNN_LAUNCH_CHECK("sb_offsets_kernel");
        if (out_nnz_host != nullptr) {
            GNN_HIP(hipMemcpyAsync(out_nnz_host, out_nnz, sizeof(int64_t), hipMemcpyDeviceToHost, stream));
            GNN_HIP(hipStreamSynchronize(stream));
        }
        return GNN_OK;
    }
    GNN_REQUIRE(out_capacity >= 0, GNN_ERR_INVALID_ARG, "out_capacity < 0");
    if (n_targets > 0) {
        // seed + hop is mixed once on the host side of the launch (same function as on the device)
        uint64_t x = seed + (uint64_t)hops;
        x += 0x9E3779B97F4A7C15ull;
        x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
        x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
        x = x ^ (x >> 31);
        sb_fill_kernel<<<wave_grid, 256, 0, stream>>>(g->row_ptr, g->col_idx, g->n_rows, target_bitmap, targets, n_targets, fanout, x,
                                                      out_row_ptr, out_col_idx, out_capacity);
        GNN_LAUNCH_CHECK("sb_fill_kernel");
    }
    return GNN_OK;
}
