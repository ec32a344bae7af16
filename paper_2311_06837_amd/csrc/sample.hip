// Expansion-aware sampling, boundary only (paper section 5.3): dependencies between inner
// (target) vertices stay whole; of the neighbours that lie outside the target set each
// target keeps at most `fanout`.  The choice is a seeded counter-based hash of the edge
// (no generator state, no dependence on thread order): the `fanout` smallest (key, id) win.
//
// Sixteen lanes per target row.  Count pass: ballots over the row give |row in T| and the
// number of outside neighbours; a three-kernel scan turns counts into row offsets.  Fill
// pass: when a row has more than `fanout` outside neighbours its lanes find the fanout-th
// smallest (key, id) by `fanout` rounds of "smallest pair above the previous one" (the row
// is re-read from cache each round), then emit the row in its original ascending order
// through a ballot-prefix compaction.  Bound: HBM (one streaming read of the target rows).
#include "common.h"
#include "hashkey.h"
#include "scan.h"

namespace gnnhot {

// Sixteen lanes per target row, four rows per wavefront (the paper's graphs have 15-50 neighbours
// per vertex).  Loops run to the longest row of the wavefront so that ballots and shuffles stay
// convergent; shorter rows are predicated off.
constexpr int kSbLanes = 16;

__device__ __forceinline__ uint32_t group_ballot(bool p, int sub) {
    return (uint32_t)((__ballot(p) >> (sub * kSbLanes)) & 0xffffu);
}

__device__ __forceinline__ int wave_max_over_groups(int x) {
    x = max(x, __shfl_xor(x, 16, kWave));
    return max(x, __shfl_xor(x, 32, kWave));
}

__global__ __launch_bounds__(256) void sb_count_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                                                       int32_t n, const uint32_t* __restrict__ tbits,
                                                       const int32_t* __restrict__ targets, int32_t n_targets, int32_t fanout,
                                                       int32_t* __restrict__ counts) {
    const int lane = lane_id(), sub = lane / kSbLanes, sl = lane % kSbLanes;
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kSbLanes;
    int32_t s = 0, e = 0;
    if (i < n_targets) {
        const int32_t v = targets[i];
        if (v >= 0 && v < n) {
            s = row_ptr[v];
            e = row_ptr[v + 1];
        }
    }
    const int len_max = wave_max_over_groups(e - s);
    int32_t n_in = 0, n_ext = 0;
    if (len_max <= 4 * kSbLanes) {  // all four loads of a lane in flight together
        int32_t ru[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int32_t p = s + r * kSbLanes + sl;
            ru[r] = p < e ? col_idx[p] : 0;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const bool valid = s + r * kSbLanes + sl < e;
            const bool inner = valid && in_set(tbits, ru[r]);
            n_in += __popc(group_ballot(inner, sub));
            n_ext += __popc(group_ballot(valid && !inner, sub));
        }
    } else
    for (int32_t off = 0; off < len_max; off += kSbLanes) {
        const int32_t p = s + off + sl;
        const bool valid = p < e;
        const bool inner = valid && in_set(tbits, col_idx[p]);
        n_in += __popc(group_ballot(inner, sub));
        n_ext += __popc(group_ballot(valid && !inner, sub));
    }
    if (sl == 0 && i < n_targets) counts[i] = n_in + (n_ext < fanout ? n_ext : fanout);
}


__global__ __launch_bounds__(256) void sb_fill_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                                                      int32_t n, const uint32_t* __restrict__ tbits,
                                                      const int32_t* __restrict__ targets, int32_t n_targets, int32_t fanout,
                                                      uint64_t seed_hop_mixed, const int32_t* __restrict__ out_row_ptr,
                                                      int32_t* __restrict__ out_col_idx, int64_t capacity) {
    const int lane = lane_id(), sub = lane / kSbLanes, sl = lane % kSbLanes;
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kSbLanes;
    int32_t v = 0, s = 0, e = 0;
    if (i < n_targets) {
        v = targets[i];
        if (v >= 0 && v < n) {
            s = row_ptr[v];
            e = row_ptr[v + 1];
        }
    }
    const int len_max = wave_max_over_groups(e - s);

    if (len_max <= 4 * kSbLanes) {
        // Fast path (every row of the wavefront has at most 64 entries): each lane holds up to four
        // entries of its row in registers, so the selection rounds need no further memory traffic.
        int32_t ru[4];
        uint64_t rk[4];
        int rf[4];  // 0: no entry, 1: neighbour inside the target set, 2: outside
        int32_t n_out = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int32_t p = s + r * kSbLanes + sl;
            ru[r] = p < e ? col_idx[p] : 0;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int32_t p = s + r * kSbLanes + sl;
            rf[r] = p < e ? (in_set(tbits, ru[r]) ? 1 : 2) : 0;
            rk[r] = rf[r] == 2 ? edge_key(seed_hop_mixed, (uint64_t)v, (uint64_t)ru[r]) : ~0ull;
            n_out += __popc(group_ballot(rf[r] == 2, sub));
        }
        uint64_t tk = ~0ull;
        int32_t tu = 0x7fffffff;
        if (fanout == 0) {
            tk = 0ull;
            tu = -1;
        }
        const bool want = fanout > 0 && n_out > fanout;
        if (__ballot(want) != 0ull) {
            uint64_t prev_k = 0ull;
            int32_t prev_u = -1;
            for (int32_t round = 0; round < fanout; ++round) {
                uint64_t best_k = ~0ull;
                int32_t best_u = 0x7fffffff;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (rf[r] == 2 && pair_less(prev_k, prev_u, rk[r], ru[r]) && pair_less(rk[r], ru[r], best_k, best_u)) {
                        best_k = rk[r];
                        best_u = ru[r];
                    }
                }
#pragma unroll
                for (int d = kSbLanes / 2; d >= 1; d >>= 1) {
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
            if (want) {
                tk = prev_k;
                tu = prev_u;
            }
        }
        int64_t at = i < n_targets ? (int64_t)out_row_ptr[i] : 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const bool keep = rf[r] == 1 || (rf[r] == 2 && !pair_less(tk, tu, rk[r], ru[r]));
            const uint32_t m = group_ballot(keep, sub);
            const int64_t my = at + __popc(m & ((1u << sl) - 1u));
            if (keep && my < capacity) out_col_idx[my] = ru[r];
            at += __popc(m);
        }
        return;
    }

    int32_t n_ext = 0;
    for (int32_t off = 0; off < len_max; off += kSbLanes) {
        const int32_t p = s + off + sl;
        n_ext += __popc(group_ballot(p < e && !in_set(tbits, col_idx[p]), sub));
    }
    // threshold pair: outside neighbours with (key, id) <= (thr_k, thr_u) are kept
    uint64_t thr_k = ~0ull;
    int32_t thr_u = 0x7fffffff;
    if (fanout == 0) {
        thr_k = 0ull;
        thr_u = -1;  // nothing is <= (0, -1): ids are non-negative
    }
    const bool need = fanout > 0 && n_ext > fanout;  // uniform over the 16-lane group
    if (__ballot(need) != 0ull) {                     // uniform over the wavefront
        uint64_t prev_k = 0ull;
        int32_t prev_u = -1;
        for (int32_t round = 0; round < fanout; ++round) {
            uint64_t best_k = ~0ull;
            int32_t best_u = 0x7fffffff;
            if (need) {
                for (int32_t p = s + sl; p < e; p += kSbLanes) {
                    const int32_t u = col_idx[p];
                    if (in_set(tbits, u)) continue;
                    const uint64_t k = edge_key(seed_hop_mixed, (uint64_t)v, (uint64_t)u);
                    if (pair_less(prev_k, prev_u, k, u) && pair_less(k, u, best_k, best_u)) {
                        best_k = k;
                        best_u = u;
                    }
                }
            }
#pragma unroll
            for (int d = kSbLanes / 2; d >= 1; d >>= 1) {
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
        if (need) {
            thr_k = prev_k;
            thr_u = prev_u;
        }
    }

    int64_t pos = i < n_targets ? (int64_t)out_row_ptr[i] : 0;
    for (int32_t off = 0; off < len_max; off += kSbLanes) {
        const int32_t p = s + off + sl;
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
        const uint32_t m = group_ballot(keep, sub);
        const int64_t my = pos + __popc(m & ((1u << sl) - 1u));
        if (keep && my < capacity) out_col_idx[my] = u;
        pos += __popc(m);
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
    const int32_t n_blocks = offsets_scan_blocks(n_targets);
    WsCarver carve(ws);
    int32_t* counts = carve.take<int32_t>((size_t)n_targets + 1);
    int32_t* sums = carve.take<int32_t>((size_t)n_blocks + 1);
    bool query;
    GNN_CHECK(ws_protocol(ws, ws_bytes, carve.used, &query));
    if (query) return GNN_OK;
    GNN_REQUIRE(out_row_ptr != nullptr, GNN_ERR_INVALID_ARG, "out_row_ptr is NULL");
    GNN_REQUIRE(n_targets == 0 || (targets != nullptr && target_bitmap != nullptr), GNN_ERR_INVALID_ARG, "targets / bitmap is NULL");
    const int wave_grid = grid_for((int64_t)n_targets * kSbLanes, 256, 1 << 30);

    if (out_col_idx == nullptr) {  // count pass
        GNN_REQUIRE(out_nnz != nullptr, GNN_ERR_INVALID_ARG, "out_nnz is NULL");
        if (n_targets > 0) {
            sb_count_kernel<<<wave_grid, 256, 0, stream>>>(g->row_ptr, g->col_idx, g->n_rows, target_bitmap, targets, n_targets, fanout,
                                                           counts);
            GNN_LAUNCH_CHECK("sb_count_kernel");
        }
        GNN_CHECK(counts_to_offsets(counts, n_targets, sums, out_row_ptr, out_nnz, stream));
        if (out_nnz_host != nullptr) {
            GNN_HIP(hipMemcpyAsync(out_nnz_host, out_nnz, sizeof(int64_t), hipMemcpyDeviceToHost, stream));
            GNN_HIP(hipStreamSynchronize(stream));
        }
        return GNN_OK;
    }
    GNN_REQUIRE(out_capacity >= 0, GNN_ERR_INVALID_ARG, "out_capacity < 0");
    if (n_targets > 0) {
        // seed + hop is mixed once on the host side of the launch (same function as on the device)
        const uint64_t x = mix64(seed + (uint64_t)hops);
        sb_fill_kernel<<<wave_grid, 256, 0, stream>>>(g->row_ptr, g->col_idx, g->n_rows, target_bitmap, targets, n_targets, fanout, x,
                                                      out_row_ptr, out_col_idx, out_capacity);
        GNN_LAUNCH_CHECK("sb_fill_kernel");
    }
    return GNN_OK;
}
