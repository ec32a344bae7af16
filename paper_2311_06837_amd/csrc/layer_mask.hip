// Layer-wise sampling as a per-layer edge mask (paper section 5.2: for layer-wise sampling methods the maskings are
// generated per layer and the layer aggregates through them).  The one-hop graph is never rebuilt: a layer's mask is
// one bit per CSR entry, which the aggregation kernels test next to their dist filter.
//
//   lm_mask_kernel       sixteen lanes per listed row (the boundary sampler's scheme): a row's keep decision is
//                        "(key, id) <= threshold pair".  A tile of sixteen consecutive entries becomes one 16-bit
//                        ballot that lane 0 ORs into the bitmap (at most two words), so the result does not depend
//                        on which group runs first.  The threshold rule has a fixed pair and takes this kernel for
//                        every row; the fanout rule takes it for rows of up to 64 entries, whose ids and keys stay in
//                        registers (four per lane) while `fanout` rounds of min-above-previous find the row's pair.
//   lm_fanout_long_kernel  the fanout rule for longer rows, a wavefront per row: one pass over the row with a bounded
//                        list of pairs in LDS (when it is full it is cut down to its `fanout` smallest, and from then
//                        on only pairs below the largest of those are listed), then one more pass that writes the bits.
//   lm_transpose_kernel  the same mask in the positions of the transposed graph (backward aggregation): entry q =
//                        (row u, column v) of the transposed graph looks up u in row v of the graph by binary search.
//   lm_mask_t_kernel     the fast way to the same transposed mask: both rules are "(key, id) <= the row's threshold
//                        pair", so with the pairs of the forward rows kept (12 bytes per row) an entry of the
//                        transposed graph is decided by one hash and one random 12-byte read.
// Bound: HBM (one pass over the listed rows; the generic transposition adds log2(row length) cached probes per entry).
#include "common.h"
#include "hashkey.h"

namespace gnnhot {

constexpr int kLmLanes = 16;

__device__ __forceinline__ uint32_t lm_group_ballot(bool p, int sub) { return (uint32_t)((__ballot(p) >> (sub * kLmLanes)) & 0xffffu); }

// ORs the 16 bits `m` (bit i = entry p0 + i) into the bitmap; called by one lane of the group
__device__ __forceinline__ void lm_or_bits(uint32_t* __restrict__ bits, int64_t p0, uint32_t m) {
    if (m == 0u) return;
    const int sh = (int)(p0 & 31);
    atomicOr(&bits[p0 >> 5], m << sh);
    if (sh > 16 && (m >> (32 - sh)) != 0u) atomicOr(&bits[(p0 >> 5) + 1], m >> (32 - sh));
}

constexpr int kLmShortRow = 64;    // fanout rule: rows up to this length stay in registers, longer ones get a wavefront
constexpr int kLmListCap = 1024;   // pairs a wavefront lists in LDS

__global__ __launch_bounds__(256) void lm_mask_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                                                      const int32_t* __restrict__ rows, int32_t n_active, int32_t rule, int32_t fanout,
                                                      uint64_t threshold, uint64_t seed_layer_mixed, uint32_t* __restrict__ bits,
                                                      int32_t* __restrict__ kept_len, uint64_t* __restrict__ row_thr_key,
                                                      int32_t* __restrict__ row_thr_id) {
    constexpr int kPerLane = kLmShortRow / kLmLanes;
    const int lane = lane_id(), sub = lane / kLmLanes, sl = lane % kLmLanes;
    const int64_t groups = ((int64_t)gridDim.x * blockDim.x) / kLmLanes;
    // the loop bound is uniform over the wavefront: its four groups take consecutive rows
    for (int64_t base = (((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6) * 4; base < n_active; base += groups) {
        const int64_t i = base + sub;
        int32_t v = 0, s = 0, e = 0;
        bool mine = i < n_active;
        if (mine) {
            v = rows ? rows[i] : (int32_t)i;
            s = row_ptr[v];
            e = row_ptr[v + 1];
        }
        // pairs (key, id) <= (thr_k, thr_u) are kept
        uint64_t thr_k = threshold;
        int32_t thr_u = 0x7fffffff;
        int32_t kept = 0;
        if (rule == GNN_LAYER_MASK_FANOUT) {   // uniform over the grid
            if (e - s > kLmShortRow) {         // lm_fanout_long_kernel takes this row
                mine = false;
                e = s;
            }
            thr_k = ~0ull;
            if (fanout == 0) {
                thr_k = 0ull;
                thr_u = -1;  // nothing is <= (0, -1): ids are non-negative
            }
            int32_t u[kPerLane];
            uint64_t key[kPerLane];
#pragma unroll
            for (int j = 0; j < kPerLane; ++j) {
                const int32_t p = s + j * kLmLanes + sl;
                u[j] = p < e ? col_idx[p] : -1;
                key[j] = u[j] >= 0 ? edge_key(seed_layer_mixed, (uint64_t)v, (uint64_t)u[j]) : ~0ull;
            }
            const bool need = fanout > 0 && e - s > fanout;  // uniform over the 16-lane group
            if (__ballot(need) != 0ull) {                     // uniform over the wavefront
                uint64_t prev_k = 0ull;
                int32_t prev_u = -1;
                for (int32_t round = 0; round < fanout; ++round) {
                    uint64_t best_k = ~0ull;
                    int32_t best_u = 0x7fffffff;
#pragma unroll
                    for (int j = 0; j < kPerLane; ++j) {
                        if (u[j] >= 0 && pair_less(prev_k, prev_u, key[j], u[j]) && pair_less(key[j], u[j], best_k, best_u)) {
                            best_k = key[j];
                            best_u = u[j];
                        }
                    }
#pragma unroll
                    for (int d = kLmLanes / 2; d >= 1; d >>= 1) {
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
#pragma unroll
            for (int j = 0; j < kPerLane; ++j) {
                const bool keep = u[j] >= 0 && !pair_less(thr_k, thr_u, key[j], u[j]);
                const uint32_t m = lm_group_ballot(keep, sub);
                kept += __popc(m);
                if (sl == 0) lm_or_bits(bits, (int64_t)s + j * kLmLanes, m);
            }
        } else {
            int len_max = e - s;
            len_max = max(len_max, __shfl_xor(len_max, 16, kWave));
            len_max = max(len_max, __shfl_xor(len_max, 32, kWave));
            for (int32_t off = 0; off < len_max; off += kLmLanes) {
                const int32_t p = s + off + sl;
                bool keep = false;
                if (p < e) {
                    const int32_t u = col_idx[p];
                    keep = !pair_less(thr_k, thr_u, edge_key(seed_layer_mixed, (uint64_t)v, (uint64_t)u), u);
                }
                const uint32_t m = lm_group_ballot(keep, sub);
                kept += __popc(m);
                if (sl == 0) lm_or_bits(bits, (int64_t)s + off, m);
            }
        }
        if (sl == 0 && mine) {
            kept_len[v] = kept;
            if (row_thr_key) {
                row_thr_key[v] = thr_k;
                row_thr_id[v] = thr_u;
            }
        }
    }
}

// Fanout rule, rows longer than kLmShortRow: one wavefront per listed row.  Pass 1 finds the row's threshold pair
// with a bounded list (see the head of the file; a fanout within 64 of the list's capacity - the list could not be
// cut down far enough to take the next 64 entries - finds it by `fanout` rounds over the row itself); pass 2 reads
// the row again and writes its bits, sixteen entries per atomic.
__global__ __launch_bounds__(256) void lm_fanout_long_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                                                             const int32_t* __restrict__ rows, int32_t n_active, int32_t fanout,
                                                             uint64_t seed_layer_mixed, uint32_t* __restrict__ bits,
                                                             int32_t* __restrict__ kept_len, uint64_t* __restrict__ row_thr_key,
                                                             int32_t* __restrict__ row_thr_id) {
    __shared__ uint64_t s_key[4][kLmListCap];
    __shared__ int32_t s_id[4][kLmListCap];
    const int lane = lane_id(), wave = (int)(threadIdx.x >> 6);
    uint64_t* key = s_key[wave];
    int32_t* id = s_id[wave];
    const uint64_t lanes_below = (1ull << lane) - 1ull;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const bool streaming = fanout <= kLmListCap - kWave;
    for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; i < n_active; i += waves) {   // uniform over the wave
        const int32_t v = rows ? rows[i] : (int32_t)i;
        const int32_t s = row_ptr[v], e = row_ptr[v + 1];
        if (e - s <= kLmShortRow) continue;
        uint64_t thr_k = ~0ull;   // pairs above (thr_k, thr_u) are out
        int32_t thr_u = 0x7fffffff;
        if (fanout == 0) {
            thr_k = 0ull;
            thr_u = -1;
        } else if (e - s > fanout && streaming) {
            int32_t n_list = 0;
            for (int32_t p = s; p < e; p += kWave) {
                const int32_t q = p + lane;
                const int32_t u = q < e ? col_idx[q] : 0;
                const uint64_t k = q < e ? edge_key(seed_layer_mixed, (uint64_t)v, (uint64_t)u) : 0ull;
                bool take = q < e && !pair_less(thr_k, thr_u, k, u);
                uint64_t mask = __ballot(take);
                if (n_list + __popcll(mask) > kLmListCap) {   // uniform: cut the list down to its fanout smallest
                    wave_lds_sync();
                    wave_list_kth(key, id, n_list, fanout, lane, thr_k, thr_u);
                    n_list = wave_list_keep_below(key, id, n_list, thr_k, thr_u, lane);
                    take = q < e && !pair_less(thr_k, thr_u, k, u);
                    mask = __ballot(take);
                }
                if (take) {
                    const int32_t pos = n_list + __popcll(mask & lanes_below);
                    key[pos] = k;
                    id[pos] = u;
                }
                n_list += __popcll(mask);
            }
            wave_lds_sync();
            if (n_list > fanout) wave_list_kth(key, id, n_list, fanout, lane, thr_k, thr_u);
            wave_lds_sync();   // the list is read before the next row overwrites it
        } else if (e - s > fanout) {
            uint64_t prev_k = 0ull;
            int32_t prev_u = -1;
            for (int32_t round = 0; round < fanout; ++round) {
                uint64_t best_k = ~0ull;
                int32_t best_u = 0x7fffffff;
                for (int32_t p = s + lane; p < e; p += kWave) {
                    const int32_t u = col_idx[p];
                    const uint64_t k = edge_key(seed_layer_mixed, (uint64_t)v, (uint64_t)u);
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
        int32_t kept = 0;
        for (int32_t p = s; p < e; p += kWave) {
            const int32_t q = p + lane;
            bool keep = false;
            if (q < e) {
                const int32_t u = col_idx[q];
                keep = !pair_less(thr_k, thr_u, edge_key(seed_layer_mixed, (uint64_t)v, (uint64_t)u), u);
            }
            const uint64_t m = __ballot(keep);
            kept += __popcll(m);
            if (lane < 4) lm_or_bits(bits, (int64_t)p + 16 * lane, (uint32_t)((m >> (16 * lane)) & 0xffffull));
        }
        if (lane == 0) {
            kept_len[v] = kept;
            if (row_thr_key) {
                row_thr_key[v] = thr_k;
                row_thr_id[v] = thr_u;
            }
        }
    }
}

// The mask of a layer in the positions of the transposed graph, from the per-row threshold pairs the forward pass
// left: entry q = (row u, column v) of the transposed graph is the forward entry (v <- u), kept iff
// (key(v, u), u) <= (row_thr_key[v], row_thr_id[v]).  One random 12-byte read per entry instead of a binary search.
__global__ __launch_bounds__(256) void lm_mask_t_kernel(int32_t n_t, const int32_t* __restrict__ rpT, const int32_t* __restrict__ ciT,
                                                        const uint64_t* __restrict__ row_thr_key, const int32_t* __restrict__ row_thr_id,
                                                        uint64_t seed_layer_mixed, uint32_t* __restrict__ keep_t) {
    const int lane = lane_id(), sub = lane / kLmLanes, sl = lane % kLmLanes;
    const int64_t groups = ((int64_t)gridDim.x * blockDim.x) / kLmLanes;
    for (int64_t base = (((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6) * 4; base < n_t; base += groups) {
        const int64_t u = base + sub;
        int32_t s = 0, e = 0;
        if (u < n_t) {
            s = rpT[u];
            e = rpT[u + 1];
        }
        int len_max = e - s;
        len_max = max(len_max, __shfl_xor(len_max, 16, kWave));
        len_max = max(len_max, __shfl_xor(len_max, 32, kWave));
        for (int32_t off = 0; off < len_max; off += kLmLanes) {
            const int32_t q = s + off + sl;
            bool bit = false;
            if (q < e) {
                const int32_t v = ciT[q];
                bit = !pair_less(row_thr_key[v], row_thr_id[v], edge_key(seed_layer_mixed, (uint64_t)v, (uint64_t)u), (int32_t)u);
            }
            const uint32_t m = lm_group_ballot(bit, sub);
            if (sl == 0) lm_or_bits(keep_t, (int64_t)s + off, m);
        }
    }
}

// thresholds of the rows that are not listed: nothing is <= (0, -1)
__global__ __launch_bounds__(256) void lm_thr_init_kernel(uint64_t* __restrict__ k, int32_t* __restrict__ u, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        k[i] = 0ull;
        u[i] = -1;
    }
}

__global__ __launch_bounds__(256) void lm_transpose_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                                                           const uint32_t* __restrict__ keep, int32_t n_t,
                                                           const int32_t* __restrict__ rpT, const int32_t* __restrict__ ciT,
                                                           uint32_t* __restrict__ keep_t) {
    const int lane = lane_id(), sub = lane / kLmLanes, sl = lane % kLmLanes;
    const int64_t groups = ((int64_t)gridDim.x * blockDim.x) / kLmLanes;
    for (int64_t base = (((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6) * 4; base < n_t; base += groups) {
        const int64_t u = base + sub;
        int32_t s = 0, e = 0;
        if (u < n_t) {
            s = rpT[u];
            e = rpT[u + 1];
        }
        int len_max = e - s;
        len_max = max(len_max, __shfl_xor(len_max, 16, kWave));
        len_max = max(len_max, __shfl_xor(len_max, 32, kWave));
        for (int32_t off = 0; off < len_max; off += kLmLanes) {
            const int32_t q = s + off + sl;
            bool bit = false;
            if (q < e) {
                const int32_t v = ciT[q];
                int32_t lo = row_ptr[v], hi = row_ptr[v + 1];  // first position of row v whose column is >= u
                while (lo < hi) {
                    const int32_t mid = lo + ((hi - lo) >> 1);
                    if (col_idx[mid] < (int32_t)u) lo = mid + 1;
                    else hi = mid;
                }
                if (lo < row_ptr[v + 1] && col_idx[lo] == (int32_t)u) bit = (keep[lo >> 5] >> (lo & 31)) & 1u;
            }
            const uint32_t m = lm_group_ballot(bit, sub);
            if (sl == 0) lm_or_bits(keep_t, (int64_t)s + off, m);
        }
    }
}

}  // namespace gnnhot

using namespace gnnhot;

extern "C" int32_t gnn_layer_edge_mask(const gnn_csr* g, const int32_t* rows, int32_t n_active, int32_t rule, int32_t fanout,
                                       uint64_t threshold, uint64_t seed, int32_t layer, uint32_t* edge_keep, int32_t* kept_len,
                                       uint64_t* row_thr_key, int32_t* row_thr_id, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    GNN_CHECK(check_csr(g, "g"));
    GNN_REQUIRE(n_active >= 0, GNN_ERR_INVALID_ARG, "negative row count");
    GNN_REQUIRE(rows != nullptr || n_active <= g->n_rows, GNN_ERR_SHAPE, "n_active %d exceeds n_rows %d", n_active, g->n_rows);
    GNN_REQUIRE(rule == GNN_LAYER_MASK_THRESHOLD || rule == GNN_LAYER_MASK_FANOUT, GNN_ERR_INVALID_ARG, "unknown mask rule %d", rule);
    GNN_REQUIRE(fanout >= 0, GNN_ERR_INVALID_ARG, "fanout < 0");
    GNN_REQUIRE(layer >= 0, GNN_ERR_INVALID_ARG, "layer < 0");
    const int64_t n_words = (g->nnz + 31) / 32;
    GNN_REQUIRE(n_words == 0 || edge_keep != nullptr, GNN_ERR_INVALID_ARG, "edge_keep is NULL");
    GNN_REQUIRE(n_active == 0 || kept_len != nullptr, GNN_ERR_INVALID_ARG, "kept_len is NULL");
    GNN_REQUIRE((row_thr_key == nullptr) == (row_thr_id == nullptr), GNN_ERR_INVALID_ARG, "row_thr_key and row_thr_id go together");
    if (row_thr_key && g->n_rows > 0) {
        lm_thr_init_kernel<<<grid_for(g->n_rows, 256, 4096), 256, 0, stream>>>(row_thr_key, row_thr_id, g->n_rows);
        GNN_LAUNCH_CHECK("lm_thr_init_kernel");
    }
    if (n_words > 0) {
        fill_kernel<uint32_t><<<grid_for(n_words, 256, 4096), 256, 0, stream>>>(edge_keep, n_words, 0u);
        GNN_LAUNCH_CHECK("fill_kernel");
    }
    if (n_active > 0) {
        lm_mask_kernel<<<grid_for((int64_t)n_active * kLmLanes, 256, 1 << 15), 256, 0, stream>>>(
            g->row_ptr, g->col_idx, rows, n_active, rule, fanout, threshold, mix64(seed + (uint64_t)layer), edge_keep, kept_len, row_thr_key,
            row_thr_id);
        GNN_LAUNCH_CHECK("lm_mask_kernel");
        if (rule == GNN_LAYER_MASK_FANOUT) {
            lm_fanout_long_kernel<<<grid_for((int64_t)n_active * kWave, 256, 4096), 256, 0, stream>>>(
                g->row_ptr, g->col_idx, rows, n_active, fanout, mix64(seed + (uint64_t)layer), edge_keep, kept_len, row_thr_key, row_thr_id);
            GNN_LAUNCH_CHECK("lm_fanout_long_kernel");
        }
    }
    return GNN_OK;
}

extern "C" int32_t gnn_transpose_edge_mask(const gnn_csr* g, const gnn_csr* gT, const uint32_t* keep, uint32_t* keep_t, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    GNN_CHECK(check_csr(g, "g"));
    GNN_CHECK(check_csr(gT, "gT"));
    GNN_REQUIRE((g->flags & GNN_CSR_SORTED_COLUMNS) != 0, GNN_ERR_UNSUPPORTED, "g must promise sorted columns");
    GNN_REQUIRE(gT->n_rows == g->n_cols && gT->n_cols == g->n_rows, GNN_ERR_SHAPE, "gT is not shaped like the transpose of g");
    const int64_t n_words = (gT->nnz + 31) / 32;
    GNN_REQUIRE(n_words == 0 || (keep != nullptr && keep_t != nullptr), GNN_ERR_INVALID_ARG, "keep or keep_t is NULL");
    if (n_words > 0) {
        fill_kernel<uint32_t><<<grid_for(n_words, 256, 4096), 256, 0, stream>>>(keep_t, n_words, 0u);
        GNN_LAUNCH_CHECK("fill_kernel");
        lm_transpose_kernel<<<grid_for((int64_t)gT->n_rows * kLmLanes, 256, 1 << 15), 256, 0, stream>>>(
            g->row_ptr, g->col_idx, keep, gT->n_rows, gT->row_ptr, gT->col_idx, keep_t);
        GNN_LAUNCH_CHECK("lm_transpose_kernel");
    }
    return GNN_OK;
}

extern "C" int32_t gnn_layer_edge_mask_transposed(const gnn_csr* gT, const uint64_t* row_thr_key, const int32_t* row_thr_id, uint64_t seed,
                                                  int32_t layer, uint32_t* keep_t, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    GNN_CHECK(check_csr(gT, "gT"));
    GNN_REQUIRE(layer >= 0, GNN_ERR_INVALID_ARG, "layer < 0");
    const int64_t n_words = (gT->nnz + 31) / 32;
    GNN_REQUIRE(n_words == 0 || (row_thr_key && row_thr_id && keep_t), GNN_ERR_INVALID_ARG, "row_thr_key, row_thr_id or keep_t is NULL");
    if (n_words > 0) {
        fill_kernel<uint32_t><<<grid_for(n_words, 256, 4096), 256, 0, stream>>>(keep_t, n_words, 0u);
        GNN_LAUNCH_CHECK("fill_kernel");
        lm_mask_t_kernel<<<grid_for((int64_t)gT->n_rows * kLmLanes, 256, 1 << 15), 256, 0, stream>>>(
            gT->n_rows, gT->row_ptr, gT->col_idx, row_thr_key, row_thr_id, mix64(seed + (uint64_t)layer), keep_t);
        GNN_LAUNCH_CHECK("lm_mask_t_kernel");
    }
    return GNN_OK;
}
