// Extraction of the partition's one-hop graph (paper section 6, figure 7c step 1: the vertices the partition
// depends on are collected outwards from its own vertices; section 5.3.1: the sub-graph is then built on what the
// traversal reached), and the matching gather of the feature rows.
//
// Input is what gnn_build_active_sets leaves for the UNPARTITIONED graph: the traversed vertices in ring order
// (sorted by (distance from the targets, id)) and dist[].  They become the local vertices 0 .. n_local-1 in that
// order, so every per-layer active set R_l of the local graph is a prefix of the numbering (targets first), and the
// local graph keeps every edge of the graph between two traversed vertices (vertex-induced sub-graph).
//
// Mapping to CDNA4.  Integer work, HBM-bound: each local row reads its global row once per pass (4 bytes per entry)
// and probes new_id[] / dist[] (4 bytes, random; both arrays are L2-resident for the partition sizes in question).
// A group of 16 lanes owns a row.  Because the numbering is (distance, id) and a global row is ascending in id, the
// row in ascending LOCAL id is the stable partition of its kept entries by distance: one ballot-compaction pass per
// distance class (at most three classes can occur in a symmetric graph - distance d-1, d, d+1 - and the passes
// re-read a row that is already in cache), no sort, bit-exact.
//
// After boundary sampling (gnn_extract_sampled_partition) the same two kernels run with other row sources: a
// target's local row is its KEPT row (the sampler's output, addressed through a row_ptr over the full id range,
// gnn_expand_row_ptr), an outside vertex's local row is the reverse of the kept edges that reach it - found by
// scanning its row of the transposed graph and keeping the targets whose kept row contains it (binary search;
// deterministic and ascending, where a scatter of the reverse edges would need atomics and a sort).
#include "common.h"
#include "scan.h"

namespace gnnhot {

constexpr int kExLanes = 16;  // lanes per local row

__global__ __launch_bounds__(256) void ex_number_kernel(const int32_t* __restrict__ ring_ids, int32_t n_local, int32_t n,
                                                         int32_t* __restrict__ new_id) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_local) {
        const int32_t v = ring_ids[i];
        if (v >= 0 && v < n) new_id[v] = (int32_t)i;
    }
}

// Where the local row of vertex v comes from, and which of its entries stay.
//   plain:    row v of g; an entry u stays if it was traversed (new_id[u] >= 0)
//   sampled:  v a target (dist 0): row v of gs (its kept row), every entry stays;
//             v outside (dist 1): row v of gT, u stays if it is a target whose kept row contains v
struct ExSource {
    const int32_t* g_rp;   // plain: g;  sampled: gT
    const int32_t* g_ci;
    const int32_t* s_rp;   // sampled only: gs (kept rows over the full id range), else NULL
    const int32_t* s_ci;
};

__device__ __forceinline__ void ex_row(const ExSource& src, const int32_t* dist, int32_t v, int32_t n, const int32_t*& ci, int32_t& s,
                                       int32_t& e, bool& reverse) {
    s = e = 0;
    ci = src.g_ci;
    reverse = false;
    if (v < 0 || v >= n) return;
    if (src.s_rp && dist[v] == 0) {
        ci = src.s_ci;
        s = src.s_rp[v];
        e = src.s_rp[v + 1];
    } else {
        reverse = src.s_rp != nullptr;
        s = src.g_rp[v];
        e = src.g_rp[v + 1];
    }
}

// is v in the kept row of target u?  (kept rows are ascending)
__device__ __forceinline__ bool ex_kept(const ExSource& src, int32_t u, int32_t v) {
    int32_t lo = src.s_rp[u], hi = src.s_rp[u + 1];
    while (lo < hi) {
        const int32_t mid = lo + ((hi - lo) >> 1);
        const int32_t c = src.s_ci[mid];
        if (c == v) return true;
        if (c < v) lo = mid + 1;
        else hi = mid;
    }
    return false;
}

__device__ __forceinline__ bool ex_stays(const ExSource& src, const int32_t* new_id, const int32_t* dist, bool reverse, int32_t v, int32_t u) {
    if (new_id[u] < 0) return false;
    if (!reverse) return true;
    return dist[u] == 0 && ex_kept(src, u, v);
}

// counts[i] = entries of the row of ring_ids[i] that stay
__global__ __launch_bounds__(256) void ex_count_kernel(ExSource src, const int32_t* __restrict__ ring_ids, int32_t n_local, int32_t n,
                                                        const int32_t* __restrict__ new_id, const int32_t* __restrict__ dist,
                                                        int32_t* __restrict__ counts) {
    const int lane = lane_id(), sub = lane / kExLanes, sl = lane % kExLanes;
    const int64_t groups = (int64_t)gridDim.x * (blockDim.x / kExLanes);
    for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kExLanes; i < n_local; i += groups) {
        const int32_t v = ring_ids[i];
        const int32_t* col_idx;
        int32_t s, e;
        bool reverse;
        ex_row(src, dist, v, n, col_idx, s, e, reverse);
        int32_t c = 0;
        for (int32_t p = s; p < e; p += kExLanes) {
            const bool keep = p + sl < e && ex_stays(src, new_id, dist, reverse, v, col_idx[p + sl]);
            c += __popcll((__ballot(keep) >> (sub * kExLanes)) & 0xffffull);
        }
        if (sl == 0) counts[i] = c;
    }
}

// out_col_idx[out_row_ptr[i] ..] = local ids of the kept entries of global row ring_ids[i], ascending
__global__ __launch_bounds__(256) void ex_fill_kernel(ExSource src, const int32_t* __restrict__ ring_ids, int32_t n_local, int32_t n,
                                                       const int32_t* __restrict__ new_id, const int32_t* __restrict__ dist, int32_t L,
                                                       const int32_t* __restrict__ out_row_ptr, int32_t* __restrict__ out_col_idx,
                                                       int64_t capacity) {
    const int lane = lane_id(), sub = lane / kExLanes, sl = lane % kExLanes;
    const int64_t groups = (int64_t)gridDim.x * (blockDim.x / kExLanes);
    for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kExLanes; i < n_local; i += groups) {
        const int32_t v = ring_ids[i];
        const int32_t* col_idx;
        int32_t s, e;
        bool reverse;
        ex_row(src, dist, v, n, col_idx, s, e, reverse);
        int64_t out = out_row_ptr[i];
        // which distance classes occur in this row (bit d), so that empty classes cost no pass
        uint32_t classes = 0;
        for (int32_t p = s; p < e; p += kExLanes) {
            if (p + sl < e) {
                const int32_t u = col_idx[p + sl];
                if (ex_stays(src, new_id, dist, reverse, v, u)) classes |= 1u << dist[u];
            }
        }
#pragma unroll
        for (int d = 1; d < kExLanes; d <<= 1) classes |= __shfl_xor(classes, d, kWave);
        for (int d = 0; d <= L; ++d) {
            if (!((classes >> d) & 1u)) continue;  // uniform over the group
            for (int32_t p = s; p < e; p += kExLanes) {
                int32_t id = -1;
                if (p + sl < e) {
                    const int32_t u = col_idx[p + sl];
                    if (dist[u] == d && ex_stays(src, new_id, dist, reverse, v, u)) id = new_id[u];
                }
                const bool keep = id >= 0;
                const uint64_t kept = (__ballot(keep) >> (sub * kExLanes)) & 0xffffull;
                const int64_t q = out + __popcll(kept & ((1ull << sl) - 1ull));
                if (keep && q < capacity) out_col_idx[q] = id;
                out += __popcll(kept);
            }
        }
    }
}

// dst[i, 0:row_bytes) = src[ids[i], 0:row_bytes): 16 lanes per row, 16 bytes per lane and step
__global__ __launch_bounds__(256) void gather_rows_kernel(const char* __restrict__ src, int64_t src_stride, const int32_t* __restrict__ ids,
                                                           int32_t n, int32_t n_src, int64_t row_bytes, char* __restrict__ dst,
                                                           int64_t dst_stride, int vec) {
    const int sl = (int)(threadIdx.x % 16);
    const int64_t groups = (int64_t)gridDim.x * (blockDim.x / 16);
    for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / 16; i < n; i += groups) {
        const int32_t v = ids[i];
        if (v < 0 || v >= n_src) continue;
        const char* s = src + (int64_t)v * src_stride;
        char* d = dst + i * dst_stride;
        if (vec) {
            for (int64_t b = (int64_t)sl * 16; b < row_bytes; b += 256) *(uint4*)(d + b) = *(const uint4*)(s + b);
        } else {
            for (int64_t b = (int64_t)sl * 2; b < row_bytes; b += 32) *(uint16_t*)(d + b) = *(const uint16_t*)(s + b);
        }
    }
}

}  // namespace gnnhot

using namespace gnnhot;

// count pass / fill pass shared by the two extraction entry points (g: the graph whose rows are scanned; gs: kept rows)
static int32_t extract_common(const gnn_csr* g, const gnn_csr* gs, const int32_t* ring_ids, int32_t n_local, const int32_t* dist,
                              int32_t L, int32_t* new_id, int32_t* out_row_ptr, int32_t* out_col_idx, int64_t out_capacity,
                              int64_t* out_nnz, int64_t* out_nnz_host, void* ws, size_t* ws_bytes, hipStream_t stream) {
    GNN_REQUIRE(g->n_rows == g->n_cols, GNN_ERR_SHAPE, "the graph must be square (%d x %d)", g->n_rows, g->n_cols);
    GNN_REQUIRE(n_local >= 0 && n_local <= g->n_rows, GNN_ERR_INVALID_ARG, "n_local %d outside [0, %d]", n_local, g->n_rows);
    GNN_REQUIRE(L >= 1 && L <= 30, GNN_ERR_INVALID_ARG, "L = %d outside [1, 30]", L);
    WsCarver carve(ws);
    int32_t* counts = carve.take<int32_t>((size_t)n_local + 1);
    int32_t* sums = carve.take<int32_t>((size_t)offsets_scan_blocks(n_local) + 1);
    bool query;
    GNN_CHECK(ws_protocol(ws, ws_bytes, carve.used, &query));
    if (query) return GNN_OK;
    GNN_REQUIRE(new_id != nullptr && out_row_ptr != nullptr, GNN_ERR_INVALID_ARG, "new_id / out_row_ptr is NULL");
    GNN_REQUIRE(n_local == 0 || (ring_ids != nullptr && dist != nullptr), GNN_ERR_INVALID_ARG, "ring_ids / dist is NULL");
    const int group_grid = grid_for((int64_t)n_local * kExLanes, 256, 1 << 20);
    ExSource src;
    src.g_rp = g->row_ptr; src.g_ci = g->col_idx;
    src.s_rp = gs ? gs->row_ptr : nullptr; src.s_ci = gs ? gs->col_idx : nullptr;

    if (out_col_idx == nullptr) {  // count pass
        GNN_REQUIRE(out_nnz != nullptr, GNN_ERR_INVALID_ARG, "out_nnz is NULL");
        if (g->n_rows > 0) {
            fill_kernel<int32_t><<<grid_for(g->n_rows, 256, 1 << 16), 256, 0, stream>>>(new_id, g->n_rows, -1);
            GNN_LAUNCH_CHECK("fill_kernel");
        }
        if (n_local > 0) {
            ex_number_kernel<<<grid_for(n_local, 256), 256, 0, stream>>>(ring_ids, n_local, g->n_rows, new_id);
            GNN_LAUNCH_CHECK("ex_number_kernel");
            ex_count_kernel<<<group_grid, 256, 0, stream>>>(src, ring_ids, n_local, g->n_rows, new_id, dist, counts);
            GNN_LAUNCH_CHECK("ex_count_kernel");
        }
        GNN_CHECK(counts_to_offsets(counts, n_local, sums, out_row_ptr, out_nnz, stream));
        if (out_nnz_host != nullptr) {
            GNN_HIP(hipMemcpyAsync(out_nnz_host, out_nnz, sizeof(int64_t), hipMemcpyDeviceToHost, stream));
            GNN_HIP(hipStreamSynchronize(stream));
        }
        return GNN_OK;
    }
    GNN_REQUIRE(out_capacity >= 0, GNN_ERR_INVALID_ARG, "out_capacity < 0");
    if (n_local > 0) {
        ex_fill_kernel<<<group_grid, 256, 0, stream>>>(src, ring_ids, n_local, g->n_rows, new_id, dist, L, out_row_ptr, out_col_idx,
                                                       out_capacity);
        GNN_LAUNCH_CHECK("ex_fill_kernel");
    }
    return GNN_OK;
}

extern "C" int32_t gnn_extract_partition(const gnn_csr* g, const int32_t* ring_ids, int32_t n_local, const int32_t* dist, int32_t L,
                                         int32_t* new_id, int32_t* out_row_ptr, int32_t* out_col_idx, int64_t out_capacity,
                                         int64_t* out_nnz, int64_t* out_nnz_host, void* ws, size_t* ws_bytes, void* stream) {
    GNN_CHECK(check_csr(g, "g"));
    return extract_common(g, nullptr, ring_ids, n_local, dist, L, new_id, out_row_ptr, out_col_idx, out_capacity, out_nnz, out_nnz_host,
                          ws, ws_bytes, (hipStream_t)stream);
}

extern "C" int32_t gnn_extract_sampled_partition(const gnn_csr* gT, const gnn_csr* gs, const int32_t* ring_ids, int32_t n_local,
                                                 const int32_t* dist, int32_t* new_id, int32_t* out_row_ptr, int32_t* out_col_idx,
                                                 int64_t out_capacity, int64_t* out_nnz, int64_t* out_nnz_host, void* ws,
                                                 size_t* ws_bytes, void* stream) {
    GNN_CHECK(check_csr(gT, "gT"));
    GNN_CHECK(check_csr(gs, "gs"));
    GNN_REQUIRE(gs->n_rows == gT->n_rows && gs->n_cols == gT->n_cols, GNN_ERR_SHAPE, "gs (%d x %d) and gT (%d x %d) differ in shape",
                gs->n_rows, gs->n_cols, gT->n_rows, gT->n_cols);
    return extract_common(gT, gs, ring_ids, n_local, dist, 1, new_id, out_row_ptr, out_col_idx, out_capacity, out_nnz, out_nnz_host, ws,
                          ws_bytes, (hipStream_t)stream);
}

// out_row_ptr over the full id range from a row list: row ids[i] gets the length of listed row i, every other row is empty
__global__ __launch_bounds__(256) void expand_lengths_kernel(const int32_t* __restrict__ ids, int32_t n_ids,
                                                              const int32_t* __restrict__ list_row_ptr, int32_t n,
                                                              int32_t* __restrict__ counts) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_ids) {
        const int32_t v = ids[i];
        if (v >= 0 && v < n) counts[v] = list_row_ptr[i + 1] - list_row_ptr[i];
    }
}

extern "C" int32_t gnn_expand_row_ptr(int32_t n, const int32_t* ids, int32_t n_ids, const int32_t* list_row_ptr, int32_t* out_row_ptr,
                                      void* ws, size_t* ws_bytes, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    GNN_REQUIRE(n >= 0 && n_ids >= 0, GNN_ERR_INVALID_ARG, "negative size");
    WsCarver carve(ws);
    int32_t* counts = carve.take<int32_t>((size_t)n + 1);
    int32_t* sums = carve.take<int32_t>((size_t)offsets_scan_blocks(n) + 1);
    int64_t* total = carve.take<int64_t>(1);
    bool query;
    GNN_CHECK(ws_protocol(ws, ws_bytes, carve.used, &query));
    if (query) return GNN_OK;
    GNN_REQUIRE(out_row_ptr != nullptr, GNN_ERR_INVALID_ARG, "out_row_ptr is NULL");
    GNN_REQUIRE(n_ids == 0 || (ids != nullptr && list_row_ptr != nullptr), GNN_ERR_INVALID_ARG, "ids / list_row_ptr is NULL");
    if (n > 0) {
        fill_kernel<int32_t><<<grid_for(n, 256, 1 << 16), 256, 0, stream>>>(counts, n, 0);
        GNN_LAUNCH_CHECK("fill_kernel");
    }
    if (n_ids > 0) {
        expand_lengths_kernel<<<grid_for(n_ids, 256), 256, 0, stream>>>(ids, n_ids, list_row_ptr, n, counts);
        GNN_LAUNCH_CHECK("expand_lengths_kernel");
    }
    return counts_to_offsets(counts, n, sums, out_row_ptr, total, stream);
}

extern "C" int32_t gnn_gather_rows(const void* src, int64_t ld_src, int32_t n_src, const int32_t* ids, int32_t n, int32_t F,
                                   int32_t dtype, void* dst, int64_t ld_dst, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    GNN_REQUIRE(dtype == GNN_F32 || dtype == GNN_BF16, GNN_ERR_UNSUPPORTED, "unknown dtype %d", dtype);
    GNN_REQUIRE(n >= 0 && F >= 0 && n_src >= 0, GNN_ERR_INVALID_ARG, "negative size");
    GNN_REQUIRE(ld_src >= F && ld_dst >= F, GNN_ERR_SHAPE, "leading dimension smaller than F = %d", F);
    if (n == 0 || F == 0) return GNN_OK;
    GNN_REQUIRE(src != nullptr && dst != nullptr && ids != nullptr, GNN_ERR_INVALID_ARG, "src / dst / ids is NULL");
    const int64_t es = dtype == GNN_F32 ? 4 : 2;
    const int64_t row_bytes = (int64_t)F * es;
    const int vec = ((uintptr_t)src % 16 == 0) && ((uintptr_t)dst % 16 == 0) && (ld_src * es) % 16 == 0 && (ld_dst * es) % 16 == 0 &&
                    row_bytes % 16 == 0;
    gather_rows_kernel<<<grid_for((int64_t)n * 16, 256, 1 << 20), 256, 0, stream>>>((const char*)src, ld_src * es, ids, n, n_src, row_bytes,
                                                                                 (char*)dst, ld_dst * es, vec);
    GNN_LAUNCH_CHECK("gather_rows_kernel");
    return GNN_OK;
}
