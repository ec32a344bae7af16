// Expansion-aware sampling, boundary only (paper section 5.3): dependencies between inner
// (target) vertices stay whole; of the neighbours that lie outside the target set each
// target keeps at most `fanout`.  The choice is a seeded counter-based hash of the edge
// (no generator state, no dependence on thread order): the `fanout` smallest (key, id) win.
//
// Rows are handled in three length classes, so that every class keeps its whole row in registers or walks it with many
// independent loads in flight (a partition grown breadth-first holds the graph's hubs: on the 10M-vertex workload 15 %
// of the target rows are longer than 64 entries and hold 70 % of all candidates):
//   up to 64 entries    sixteen lanes per row, four entries per lane;
//   65 to 1024          one wavefront per row, sixteen entries per lane (second launch of the pass);
//   longer              one workgroup per row, which strides the row four entries per thread and step (third launch).
// The first launch is a grid-stride loop over the targets; the rows it leaves to the other two are collected in LDS
// lists and appended to the two queues with ONE global atomic per workgroup and class (one atomic per row on a single
// counter serialised the launch: 184 000 of them took 1.4 ms).  Count pass: ballots give |row in T| and the number of
// outside neighbours; a three-kernel scan turns counts into row offsets.  Fill pass: a row with more than `fanout`
// outside neighbours finds the fanout-th smallest (key, id) by `fanout` rounds of "smallest pair above the previous
// one" over its registers, then emits the row in its original ascending order through a ballot-prefix compaction.
// Which lane group, wavefront or workgroup takes a row does not matter: every row's result depends on the row alone.
// Bound: HBM (one streaming read of the target rows per pass).
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

constexpr int kSbShort = 4 * kSbLanes;   // rows up to this length stay with their sixteen lanes
constexpr int kSbMedium = 16 * kWave;    // rows up to this length get a wavefront, longer ones a workgroup
constexpr int kSbRowsPerWg = 256 / kSbLanes;   // rows one workgroup of the first launch takes per step
constexpr int kSbListCap = 1024;         // entries of a workgroup's LDS list per class; what does not fit goes out one by one

struct SbCtrl {
    int32_t n_medium;
    int32_t n_hub;
    int32_t pad[6];
};

// A workgroup's lists of the rows it leaves to the wavefront-per-row and workgroup-per-row launches.
struct SbLists {
    int32_t med[kSbListCap], hub[kSbListCap];
    int32_t n_med, n_hub, base_med, base_hub;
};

__device__ __forceinline__ void sb_lists_init(SbLists& L) {
    if (threadIdx.x == 0) L.n_med = L.n_hub = 0;
    __syncthreads();
}

// one lane per row calls this
__device__ __forceinline__ void sb_lists_push(SbLists& L, int32_t i, int32_t len, int32_t* __restrict__ medq, int32_t* __restrict__ hubq,
                                              SbCtrl* ctrl) {
    if (len <= kSbMedium) {
        const int pos = atomicAdd(&L.n_med, 1);
        if (pos < kSbListCap) L.med[pos] = i;
        else medq[atomicAdd(&ctrl->n_medium, 1)] = i;
    } else {
        const int pos = atomicAdd(&L.n_hub, 1);
        if (pos < kSbListCap) L.hub[pos] = i;
        else hubq[atomicAdd(&ctrl->n_hub, 1)] = i;
    }
}

// every thread of the workgroup calls this once, after its last push
__device__ __forceinline__ void sb_lists_flush(SbLists& L, int32_t* __restrict__ medq, int32_t* __restrict__ hubq, SbCtrl* ctrl) {
    __syncthreads();
    const int nm = L.n_med < kSbListCap ? L.n_med : kSbListCap, nh = L.n_hub < kSbListCap ? L.n_hub : kSbListCap;
    if (threadIdx.x == 0) {
        L.base_med = nm ? atomicAdd(&ctrl->n_medium, nm) : 0;
        L.base_hub = nh ? atomicAdd(&ctrl->n_hub, nh) : 0;
    }
    __syncthreads();
    for (int k = threadIdx.x; k < nm; k += blockDim.x) medq[L.base_med + k] = L.med[k];
    for (int k = threadIdx.x; k < nh; k += blockDim.x) hubq[L.base_hub + k] = L.hub[k];
}

__global__ __launch_bounds__(256) void sb_count_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                                                       int32_t n, const uint32_t* __restrict__ tbits,
                                                       const int32_t* __restrict__ targets, int32_t n_targets, int32_t fanout,
                                                       int32_t* __restrict__ counts, int32_t* __restrict__ medq,
                                                       int32_t* __restrict__ hubq, SbCtrl* ctrl) {
    __shared__ SbLists lists;
    sb_lists_init(lists);
    const int lane = lane_id(), sub = lane / kSbLanes, sl = lane % kSbLanes;
    const int grp = (int)threadIdx.x / kSbLanes;
    for (int64_t c = blockIdx.x; c * kSbRowsPerWg < n_targets; c += gridDim.x) {   // uniform over the workgroup
        const int64_t i = c * kSbRowsPerWg + grp;
        int32_t s = 0, e = 0;
        if (i < n_targets) {
            const int32_t v = targets[i];
            if (v >= 0 && v < n) {
                s = row_ptr[v];
                e = row_ptr[v + 1];
            }
        }
        const bool is_long = e - s > kSbShort;   // uniform over the 16-lane group
        if (is_long) {
            if (sl == 0) sb_lists_push(lists, (int32_t)i, e - s, medq, hubq, ctrl);
            s = e = 0;
        }
        int32_t n_in = 0, n_ext = 0;
        int32_t ru[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {  // all four loads of a lane in flight together
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
        if (sl == 0 && i < n_targets && !is_long) counts[i] = n_in + (n_ext < fanout ? n_ext : fanout);
    }
    sb_lists_flush(lists, medq, hubq, ctrl);
}


__global__ __launch_bounds__(256) void sb_fill_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                                                      int32_t n, const uint32_t* __restrict__ tbits,
                                                      const int32_t* __restrict__ targets, int32_t n_targets, int32_t fanout,
                                                      uint64_t seed_hop_mixed, const int32_t* __restrict__ out_row_ptr,
                                                      int32_t* __restrict__ out_col_idx, int64_t capacity,
                                                      int32_t* __restrict__ medq, int32_t* __restrict__ hubq, SbCtrl* ctrl) {
    __shared__ SbLists lists;
    sb_lists_init(lists);
    const int lane = lane_id(), sub = lane / kSbLanes, sl = lane % kSbLanes;
    const int grp = (int)threadIdx.x / kSbLanes;
    for (int64_t c = blockIdx.x; c * kSbRowsPerWg < n_targets; c += gridDim.x) {   // uniform over the workgroup
    const int64_t i = c * kSbRowsPerWg + grp;
    int32_t v = 0, s = 0, e = 0;
    if (i < n_targets) {
        v = targets[i];
        if (v >= 0 && v < n) {
            s = row_ptr[v];
            e = row_ptr[v + 1];
        }
    }
    if (e - s > kSbShort) {   // uniform over the 16-lane group: a wavefront or a workgroup of the later launches takes this row
        if (sl == 0) sb_lists_push(lists, (int32_t)i, e - s, medq, hubq, ctrl);
        s = e = 0;
    }
    // each lane holds up to four entries of its row in registers, so the selection rounds need no further memory traffic
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
    // threshold pair: outside neighbours with (key, id) <= (tk, tu) are kept
    uint64_t tk = ~0ull;
    int32_t tu = 0x7fffffff;
    if (fanout == 0) {
        tk = 0ull;
        tu = -1;  // nothing is <= (0, -1): ids are non-negative
    }
    const bool want = fanout > 0 && n_out > fanout;   // uniform over the 16-lane group
    if (__ballot(want) != 0ull) {                      // uniform over the wavefront
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
    }   // grid-stride loop
    sb_lists_flush(lists, medq, hubq, ctrl);
}

// ---- rows of 65 to 1024 entries: one wavefront per queued row, sixteen entries per lane, everything in registers --------
template <bool FILL>
__global__ __launch_bounds__(256) void sb_medium_rows_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                                                             const uint32_t* __restrict__ tbits, const int32_t* __restrict__ targets,
                                                             const int32_t* __restrict__ medq, const SbCtrl* __restrict__ ctrl,
                                                             int32_t fanout, uint64_t seed_hop_mixed, int32_t* __restrict__ counts,
                                                             const int32_t* __restrict__ out_row_ptr, int32_t* __restrict__ out_col_idx,
                                                             int64_t capacity) {
    constexpr int EPL = kSbMedium / kWave;   // entries per lane
    const int lane = lane_id();
    const int64_t wave_g = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const int32_t n_med = ctrl->n_medium;
    for (int64_t h = wave_g; h < n_med; h += n_waves) {   // uniform over the wavefront
        const int32_t i = medq[h];
        const int32_t v = targets[i];
        const int32_t s = row_ptr[v], e = row_ptr[v + 1];
        int32_t ru[EPL];
        int rf[EPL];  // 0: no entry, 1: neighbour inside the target set, 2: outside
#pragma unroll
        for (int r = 0; r < EPL; ++r) {
            const int32_t p = s + r * kWave + lane;
            ru[r] = p < e ? col_idx[p] : 0;
        }
        int32_t n_in = 0, n_ext = 0;
#pragma unroll
        for (int r = 0; r < EPL; ++r) {
            const int32_t p = s + r * kWave + lane;
            rf[r] = p < e ? (in_set(tbits, ru[r]) ? 1 : 2) : 0;
            n_in += __popcll(__ballot(rf[r] == 1));
            n_ext += __popcll(__ballot(rf[r] == 2));
        }
        if (!FILL) {
            if (lane == 0) counts[i] = n_in + (n_ext < fanout ? n_ext : fanout);
            continue;
        }
        uint64_t rk[EPL];
#pragma unroll
        for (int r = 0; r < EPL; ++r) rk[r] = rf[r] == 2 ? edge_key(seed_hop_mixed, (uint64_t)v, (uint64_t)ru[r]) : ~0ull;
        uint64_t tk = ~0ull;
        int32_t tu = 0x7fffffff;
        if (fanout == 0) {
            tk = 0ull;
            tu = -1;
        }
        if (fanout > 0 && n_ext > fanout) {   // uniform over the wavefront
            uint64_t prev_k = 0ull;
            int32_t prev_u = -1;
            for (int32_t round = 0; round < fanout; ++round) {
                uint64_t best_k = ~0ull;
                int32_t best_u = 0x7fffffff;
#pragma unroll
                for (int r = 0; r < EPL; ++r) {
                    if (rf[r] == 2 && pair_less(prev_k, prev_u, rk[r], ru[r]) && pair_less(rk[r], ru[r], best_k, best_u)) {
                        best_k = rk[r];
                        best_u = ru[r];
                    }
                }
#pragma unroll
                for (int d = kWave / 2; d >= 1; d >>= 1) {
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
            tk = prev_k;
            tu = prev_u;
        }
        int64_t at = out_row_ptr[i];
        const uint64_t below = (1ull << lane) - 1ull;
#pragma unroll
        for (int r = 0; r < EPL; ++r) {
            const bool keep = rf[r] == 1 || (rf[r] == 2 && !pair_less(tk, tu, rk[r], ru[r]));
            const uint64_t m = __ballot(keep);
            const int64_t my = at + __popcll(m & below);
            if (keep && my < capacity) out_col_idx[my] = ru[r];
            at += __popcll(m);
        }
    }
}


// ---- rows of more than 1024 entries: one workgroup per queued row -----------------------------------------------
// Sums of two ints over the workgroup (every thread gets them).  Two barriers.
__device__ __forceinline__ void block_sum2(int& a, int& b, int* s_a, int* s_b) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        a += __shfl_xor(a, d, kWave);
        b += __shfl_xor(b, d, kWave);
    }
    const int w = (int)(threadIdx.x >> 6);
    if (lane_id() == 0) {
        s_a[w] = a;
        s_b[w] = b;
    }
    __syncthreads();
    a = s_a[0] + s_a[1] + s_a[2] + s_a[3];
    b = s_b[0] + s_b[1] + s_b[2] + s_b[3];
    __syncthreads();
}

// Smallest (key, id) pair over the workgroup (every thread gets it).  Two barriers.
__device__ __forceinline__ void block_min_pair(uint64_t& k, int32_t& u, uint64_t* s_k, int32_t* s_u) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const uint64_t ok = __shfl_xor(k, d, kWave);
        const int32_t ou = __shfl_xor(u, d, kWave);
        if (pair_less(ok, ou, k, u)) {
            k = ok;
            u = ou;
        }
    }
    const int w = (int)(threadIdx.x >> 6);
    if (lane_id() == 0) {
        s_k[w] = k;
        s_u[w] = u;
    }
    __syncthreads();
    k = s_k[0];
    u = s_u[0];
#pragma unroll
    for (int q = 1; q < 4; ++q)
        if (pair_less(s_k[q], s_u[q], k, u)) {
            k = s_k[q];
            u = s_u[q];
        }
    __syncthreads();
}

// The same selection as the sixteen-lane kernels, for the queued rows: 256 threads stride the row, four entries per
// thread and step with all their loads (ids, then target bits) issued before the first use.  FILL false: counts[i];
// FILL true: the kept ids in ascending position order.  Which workgroup takes which row does not matter: every row's
// result depends on the row alone.
template <bool FILL>
__global__ __launch_bounds__(256) void sb_long_rows_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                                                           const uint32_t* __restrict__ tbits, const int32_t* __restrict__ targets,
                                                           const int32_t* __restrict__ hubq, const SbCtrl* __restrict__ ctrl,
                                                           int32_t fanout, uint64_t seed_hop_mixed, int32_t* __restrict__ counts,
                                                           const int32_t* __restrict__ out_row_ptr, int32_t* __restrict__ out_col_idx,
                                                           int64_t capacity) {
    __shared__ int s_a[4], s_b[4], s_part[4];
    __shared__ uint64_t s_k[4];
    __shared__ int32_t s_u[4];
    const int tid = (int)threadIdx.x;
    const int32_t n_hub = ctrl->n_hub;
    for (int32_t h = blockIdx.x; h < n_hub; h += gridDim.x) {   // uniform over the workgroup
        const int32_t i = hubq[h];
        const int32_t v = targets[i];
        const int32_t s = row_ptr[v], e = row_ptr[v + 1];
        int n_in = 0, n_ext = 0;
        for (int32_t base = s; base < e; base += 1024) {
            int32_t u[4];
            bool ok[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int32_t p = base + r * 256 + tid;
                ok[r] = p < e;
                u[r] = ok[r] ? col_idx[p] : 0;
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool inner = in_set(tbits, u[r]);     // u = 0 where the thread has no entry: a valid probe
                n_in += ok[r] && inner;
                n_ext += ok[r] && !inner;
            }
        }
        block_sum2(n_in, n_ext, s_a, s_b);
        if (!FILL) {
            if (tid == 0) counts[i] = n_in + (n_ext < fanout ? n_ext : fanout);
            continue;
        }
        uint64_t thr_k = ~0ull;
        int32_t thr_u = 0x7fffffff;
        if (fanout == 0) {
            thr_k = 0ull;
            thr_u = -1;
        }
        if (fanout > 0 && n_ext > fanout) {   // uniform over the workgroup
            uint64_t prev_k = 0ull;
            int32_t prev_u = -1;
            for (int32_t round = 0; round < fanout; ++round) {
                uint64_t best_k = ~0ull;
                int32_t best_u = 0x7fffffff;
                for (int32_t base = s; base < e; base += 1024) {
                    int32_t u[4];
                    bool ok[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int32_t p = base + r * 256 + tid;
                        ok[r] = p < e;
                        u[r] = ok[r] ? col_idx[p] : 0;
                    }
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        if (ok[r] && !in_set(tbits, u[r])) {
                            const uint64_t k = edge_key(seed_hop_mixed, (uint64_t)v, (uint64_t)u[r]);
                            if (pair_less(prev_k, prev_u, k, u[r]) && pair_less(k, u[r], best_k, best_u)) {
                                best_k = k;
                                best_u = u[r];
                            }
                        }
                    }
                }
                block_min_pair(best_k, best_u, s_k, s_u);
                prev_k = best_k;
                prev_u = best_u;
            }
            thr_k = prev_k;
            thr_u = prev_u;
        }
        int64_t pos = out_row_ptr[i];
        for (int32_t base = s; base < e; base += 256) {
            const int32_t p = base + tid;
            bool keep = false;
            int32_t u = 0;
            if (p < e) {
                u = col_idx[p];
                if (in_set(tbits, u)) keep = true;
                else keep = !pair_less(thr_k, thr_u, edge_key(seed_hop_mixed, (uint64_t)v, (uint64_t)u), u);
            }
            int total;
            const int before = block_exclusive_scan<256>(keep ? 1 : 0, s_part, &total);
            if (keep && pos + before < capacity) out_col_idx[pos + before] = u;
            pos += total;
        }
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
    int32_t* medq = carve.take<int32_t>((size_t)n_targets + 1);   // positions (in `targets`) of the rows of 65 to 1024 entries
    int32_t* hubq = carve.take<int32_t>((size_t)n_targets + 1);   // ... and of the longer ones
    SbCtrl* ctrl = carve.take<SbCtrl>(1);
    bool query;
    GNN_CHECK(ws_protocol(ws, ws_bytes, carve.used, &query));
    if (query) return GNN_OK;
    GNN_REQUIRE(out_row_ptr != nullptr, GNN_ERR_INVALID_ARG, "out_row_ptr is NULL");
    GNN_REQUIRE(n_targets == 0 || (targets != nullptr && target_bitmap != nullptr), GNN_ERR_INVALID_ARG, "targets / bitmap is NULL");
    const int wave_grid = grid_for((int64_t)n_targets * kSbLanes, 256, 4096);   // grid-stride: one queue append per workgroup
    if (n_targets > 0) {   // both passes queue their long rows afresh (workspace contents do not survive a call)
        fill_kernel<int32_t><<<1, 64, 0, stream>>>((int32_t*)ctrl, (int64_t)(sizeof(SbCtrl) / sizeof(int32_t)), 0);
        GNN_LAUNCH_CHECK("fill_kernel");
    }
    const int long_grid = 2048;   // grid-stride over the queues, whose lengths only the device knows

    if (out_col_idx == nullptr) {  // count pass
        GNN_REQUIRE(out_nnz != nullptr, GNN_ERR_INVALID_ARG, "out_nnz is NULL");
        if (n_targets > 0) {
            sb_count_kernel<<<wave_grid, 256, 0, stream>>>(g->row_ptr, g->col_idx, g->n_rows, target_bitmap, targets, n_targets, fanout,
                                                           counts, medq, hubq, ctrl);
            GNN_LAUNCH_CHECK("sb_count_kernel");
            sb_medium_rows_kernel<false><<<long_grid, 256, 0, stream>>>(g->row_ptr, g->col_idx, target_bitmap, targets, medq, ctrl, fanout,
                                                                        0ull, counts, nullptr, nullptr, 0);
            GNN_LAUNCH_CHECK("sb_medium_rows_kernel");
            sb_long_rows_kernel<false><<<long_grid, 256, 0, stream>>>(g->row_ptr, g->col_idx, target_bitmap, targets, hubq, ctrl, fanout,
                                                                      0ull, counts, nullptr, nullptr, 0);
            GNN_LAUNCH_CHECK("sb_long_rows_kernel");
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
                                                      out_row_ptr, out_col_idx, out_capacity, medq, hubq, ctrl);
        GNN_LAUNCH_CHECK("sb_fill_kernel");
        sb_medium_rows_kernel<true><<<long_grid, 256, 0, stream>>>(g->row_ptr, g->col_idx, target_bitmap, targets, medq, ctrl, fanout, x,
                                                                   nullptr, out_row_ptr, out_col_idx, out_capacity);
        GNN_LAUNCH_CHECK("sb_medium_rows_kernel");
        sb_long_rows_kernel<true><<<long_grid, 256, 0, stream>>>(g->row_ptr, g->col_idx, target_bitmap, targets, hubq, ctrl, fanout, x,
                                                                 nullptr, out_row_ptr, out_col_idx, out_capacity);
        GNN_LAUNCH_CHECK("sb_long_rows_kernel");
    }
    return GNN_OK;
}
