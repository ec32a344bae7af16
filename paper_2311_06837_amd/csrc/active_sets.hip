// Per-layer active vertex sets: level-synchronous frontier expansion from the targets
// (paper section 6, figure 7c: step 1 extracts the multi-hop dependency from the inner
// vertices, step 4 generates the per-layer mask).
//
// Data layout.  In the workspace: two bitmaps of n bits, `visited` (everything reached by the
// levels before the one being expanded, read-only while it expands) and `frontier` (the ring
// the last level found), and `seen`, ONE BYTE per vertex (`visited` plus what the level has
// found so far).  `seen` is bytes because every lane that finds a vertex marks it: a byte takes
// a plain store of 1 - whoever comes first, the byte ends up the same - where a bit needs an
// atomic OR, and a ring of a few million new vertices packs those atomics onto a few thousand
// cache lines (measured: 0.60 ms of atomics for 24 M edges that discover 2.2 M vertices).
// The byte accesses are ordinary loads and stores on purpose: a stale 0 from the vector cache
// only means one more store of the same 1 (relaxed atomic loads, which bypass that cache, were
// measured 15 to 50 % slower per construction); kernel boundaries order the levels.
// A level is: expand -> count / scan / emit, a compaction of seen & ~visited that lists the
// new ring in ascending id order without any sort, so the output does not depend on which
// wave found a vertex first; emit then brings visited up to seen.  Ring sizes stay on
// the device (hop_offsets); every kernel has a fixed grid and reads its bounds from there, so
// the whole construction is enqueued without a host round trip.
//
// A level expands in one of two directions; the sets are the same either way.
//   push  (from the frontier)  EDGE-parallel: a wavefront takes up to 64 frontier vertices, reads
//         their row bounds in one sweep, and then walks the concatenation of their rows 256
//         edges at a time (each lane finds the row of its edge by a binary search over the 64
//         prefix sums in LDS), so rows of 5 and rows of 500 entries keep all lanes busy alike
//         and every lane has four independent index loads and four bitmap probes in flight.
//         One probe of `seen` per edge; the byte is set if still clear.
//   pull  (from the unreached vertices; needs the transposed graph)  sixteen lanes per
//         unreached vertex scan its row of the transposed graph - the vertices that would
//         reach it - and stop at the first one that is in `frontier`.  Once the frontier is
//         most of the graph, nearly every edge of a push level points at a vertex that is
//         already in the set; the pull level only touches the few vertices still outside.
// The direction is chosen on the device, per level, from exact integer sums (as_plan_kernel):
// pull when the frontier's edges outnumber what a pull can touch at most, the transposed
// rows of the unreached vertices plus sixteen lanes for each of them.  Both kernels of a level
// are enqueued; the one whose turn it is not returns at once.
//
// Bound: a push level reads each edge of the frontier once (4 B, streaming) and makes one
// 1-byte probe per edge into n bytes that stay in L2: the probes, not the bytes, are what
// limits it (the L2s serve a fixed number of requests per clock).
#include "common.h"
#include "hashkey.h"
#include "scan.h"

namespace gnnhot {

constexpr int kAsWordsPerBlock = 256;   // one bitmap word per thread: 8192 vertices per block
constexpr int kAsHubDegree = 2048;      // longer rows are queued and expanded by a whole workgroup each

struct AsCtrl {
    int32_t n_hubs;
    int32_t pad;
    unsigned long long frontier_edges;   // entries of the frontier's rows (graph), this level
    unsigned long long reached_edges_t;  // entries of the transposed rows of everything reached so far
    unsigned long long pad2;
};

// True when this level runs in the pull direction.  frontier = ring `ring_prev`.  A pull touches at most the transposed
// rows of the unreached vertices, sixteen lanes at a time.
__device__ __forceinline__ bool as_pull_level(const AsCtrl* ctrl, const int64_t* __restrict__ hop_offsets, int32_t ring_prev,
                                              int64_t n, int64_t nnz_t) {
    const int64_t unreached = n - hop_offsets[ring_prev + 1];
    const int64_t unreached_edges = nnz_t - (int64_t)ctrl->reached_edges_t;
    return (int64_t)ctrl->frontier_edges > unreached_edges + 16 * unreached;
}

// Bit b of the result = byte b of the 32 bytes at p (each 0 or 1); p is 32-byte aligned.
__device__ __forceinline__ uint32_t as_mask_of_bytes(const uint8_t* __restrict__ p) {
    const uint4 a = *(const uint4*)p, b = *(const uint4*)(p + 16);
    const uint32_t x[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    uint32_t m = 0u;
#pragma unroll
    for (int k = 0; k < 8; ++k)
        m |= ((x[k] & 1u) | ((x[k] >> 7) & 2u) | ((x[k] >> 14) & 4u) | ((x[k] >> 21) & 8u)) << (4 * k);
    return m;
}

__global__ __launch_bounds__(256) void as_init_kernel(int32_t* __restrict__ dist, int32_t n, uint32_t* __restrict__ visited,
                                                      uint8_t* __restrict__ seen, int64_t nw, AsCtrl* ctrl,
                                                      int64_t* __restrict__ hop_offsets, int32_t L) {
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t v = tid; v < n; v += stride) dist[v] = -1;
    for (int64_t w = tid; w < nw; w += stride) {
        visited[w] = 0u;
        ((uint4*)seen)[2 * w] = make_uint4(0u, 0u, 0u, 0u);   // 32 bytes per bitmap word, the tail of the last word included
        ((uint4*)seen)[2 * w + 1] = make_uint4(0u, 0u, 0u, 0u);
    }
    if (tid == 0) {
        ctrl->n_hubs = 0;
        ctrl->frontier_edges = 0ull;
        ctrl->reached_edges_t = 0ull;
    }
    if (tid <= L + 1) hop_offsets[tid] = 0;
}

__global__ __launch_bounds__(256) void as_seed_kernel(const int32_t* __restrict__ targets, int32_t n_targets, int32_t n,
                                                      uint8_t* __restrict__ seen) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_targets; i += (int64_t)gridDim.x * blockDim.x) {
        int32_t v = targets[i];
        if (v >= 0 && v < n) seen[v] = 1;
    }
}

constexpr int kAsU = 8;   // edges per lane and step: their index loads, then their probes, are issued together

// Push level.  One wavefront per batch of up to 64 entries of the frontier list (grid-stride), edge-parallel inside
// (see the head of the file).  A step of a wavefront is a chain of dependent loads (row bounds, ids, probes: about
// 3 us), so what a level costs is the number of steps of its busiest wavefront: the batch is made as small as it can be
// while every batch still finds a wavefront of its own (a power of two, at least 1) - 29 000 frontier vertices of
// 490 entries each are 122 steps per wavefront in batches of 64 and 4 in batches of 4 (measured on the 8-level
// workload, 62 500 frontier vertices of 27 entries: 0.28 -> 0.08 ms for the level).
// nnz_t < 0: no transposed graph was given, every level is a push level.
__global__ __launch_bounds__(256) void as_expand_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                                                        const int32_t* __restrict__ ring_ids,
                                                        const int64_t* __restrict__ hop_offsets, int32_t ring,
                                                        uint8_t* __restrict__ seen, int32_t* __restrict__ hubq, AsCtrl* ctrl,
                                                        int32_t n, int64_t nnz_t) {
    __shared__ int32_t s_start[4][kWave];
    __shared__ int32_t s_excl[4][kWave + 1];
    if (nnz_t >= 0 && as_pull_level(ctrl, hop_offsets, ring, n, nnz_t)) return;   // uniform over the grid
    const int64_t begin = hop_offsets[ring], end = hop_offsets[ring + 1];
    const int lane = lane_id(), wave = (int)(threadIdx.x >> 6);
    int32_t* st = s_start[wave];
    int32_t* ex = s_excl[wave];
    const int64_t wave_g = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    int batch = kWave;
    while (batch > 1 && (int64_t)(batch >> 1) * n_waves >= end - begin) batch >>= 1;
    for (int64_t b = begin + wave_g * batch; b < end; b += n_waves * batch) {   // uniform over the wavefront
        const int64_t i = b + lane;
        int32_t s = 0, len = 0;
        if (lane < batch && i < end) {
            const int32_t v = ring_ids[i];
            s = row_ptr[v];
            len = row_ptr[v + 1] - s;
            if (len > kAsHubDegree) {   // a whole workgroup of the next launch takes this row
                hubq[atomicAdd(&ctrl->n_hubs, 1)] = v;
                len = 0;
            }
        }
        const int incl = wave_inclusive_scan(len);
        const int total = __shfl(incl, kWave - 1, kWave);
        wave_lds_sync();   // the previous batch has been read
        st[lane] = s;
        ex[lane] = incl - len;
        if (lane == kWave - 1) ex[kWave] = total;
        wave_lds_sync();
        for (int t0 = 0; t0 < total; t0 += kWave * kAsU) {
            int32_t u[kAsU];
            bool ok[kAsU];
#pragma unroll
            for (int j = 0; j < kAsU; ++j) {
                const int t = t0 + j * kWave + lane;
                ok[j] = t < total;
                int lo = 0, hi = kWave;   // ex[lo] <= t < ex[hi]: the row that holds edge t (empty rows are stepped over)
                if (ok[j]) {
#pragma unroll
                    for (int k = 0; k < 6; ++k) {
                        const int mid = (lo + hi) >> 1;
                        if (ex[mid] <= t) lo = mid;
                        else hi = mid;
                    }
                }
                u[j] = ok[j] ? col_idx[st[lo] + (t - ex[lo])] : 0;
            }
            uint8_t w[kAsU];
#pragma unroll
            for (int j = 0; j < kAsU; ++j) w[j] = seen[u[j]];   // u = 0 where the lane has no edge: a valid byte
#pragma unroll
            for (int j = 0; j < kAsU; ++j)
                if (ok[j] && !w[j]) seen[u[j]] = 1;
        }
    }
}

// Hub rows of a push level: the queued rows are cut into as many equal pieces as the grid has workgroups per row, a
// workgroup per piece (grid-stride), threads across the piece, kAsU entries per thread and step.  (In a pull level the
// queue is empty when this kernel runs.)
__global__ __launch_bounds__(256) void as_expand_hubs_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                                                             uint8_t* __restrict__ seen, const int32_t* __restrict__ hubq,
                                                             const AsCtrl* ctrl) {
    const int32_t n_hubs = ctrl->n_hubs;
    if (n_hubs <= 0) return;
    const int32_t parts = (int32_t)gridDim.x / n_hubs > 1 ? (int32_t)gridDim.x / n_hubs : 1;
    for (int64_t job = blockIdx.x; job < (int64_t)n_hubs * parts; job += gridDim.x) {   // uniform over the workgroup
        const int32_t v = hubq[job / parts];
        const int32_t part = (int32_t)(job % parts);
        const int64_t s0 = row_ptr[v], len = row_ptr[v + 1] - s0;
        const int32_t s = (int32_t)(s0 + len * part / parts), e = (int32_t)(s0 + len * (part + 1) / parts);
        for (int32_t base = s + (int32_t)threadIdx.x; base < e; base += 256 * kAsU) {
            int32_t u[kAsU];
            uint8_t w[kAsU];
#pragma unroll
            for (int j = 0; j < kAsU; ++j) u[j] = base + j * 256 < e ? col_idx[base + j * 256] : 0;
#pragma unroll
            for (int j = 0; j < kAsU; ++j) w[j] = seen[u[j]];
#pragma unroll
            for (int j = 0; j < kAsU; ++j)
                if (base + j * 256 < e && !w[j]) seen[u[j]] = 1;
        }
    }
}

// Exact sums the direction switch needs, over the ring the next level expands: entries of its rows (what a push
// reads) and entries of its transposed rows (added to the running total of everything reached).  Integer atomics:
// the totals do not depend on the order of the additions.
__global__ __launch_bounds__(256) void as_plan_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ row_ptr_t,
                                                      const int32_t* __restrict__ ring_ids, const int64_t* __restrict__ hop_offsets,
                                                      int32_t ring, AsCtrl* ctrl) {
    __shared__ unsigned long long s_a[4], s_b[4];
    const int64_t begin = hop_offsets[ring], end = hop_offsets[ring + 1];
    unsigned long long a = 0ull, b = 0ull;
    for (int64_t i = begin + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < end; i += (int64_t)gridDim.x * blockDim.x) {
        const int32_t v = ring_ids[i];
        a += (unsigned long long)(row_ptr[v + 1] - row_ptr[v]);
        b += (unsigned long long)(row_ptr_t[v + 1] - row_ptr_t[v]);
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        a += __shfl_xor(a, d, kWave);
        b += __shfl_xor(b, d, kWave);
    }
    if (lane_id() == 0) {
        s_a[threadIdx.x >> 6] = a;
        s_b[threadIdx.x >> 6] = b;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        a = s_a[0] + s_a[1] + s_a[2] + s_a[3];
        b = s_b[0] + s_b[1] + s_b[2] + s_b[3];
        if (a) atomicAdd(&ctrl->frontier_edges, a);
        if (b) atomicAdd(&ctrl->reached_edges_t, b);
    }
}

// Pull level.  A wavefront per bitmap word (grid-stride), sixteen lanes per vertex: for each vertex of the word that is
// not in the set yet, scan its transposed row 64 entries at a time and stop at the first entry that is in the frontier.  A lane group
// is the only writer of its vertices' bytes in this kernel.  Rows longer than kAsHubDegree go to the queue.
__global__ __launch_bounds__(256) void as_pull_kernel(const int32_t* __restrict__ row_ptr_t, const int32_t* __restrict__ col_idx_t,
                                                      int32_t n, int64_t nw, const uint32_t* __restrict__ visited,
                                                      uint8_t* __restrict__ seen, const uint32_t* __restrict__ frontier,
                                                      const int64_t* __restrict__ hop_offsets, int32_t ring, int64_t nnz_t,
                                                      int32_t* __restrict__ hubq, AsCtrl* ctrl) {
    if (!as_pull_level(ctrl, hop_offsets, ring, n, nnz_t)) return;   // uniform over the grid
    const int lane = lane_id(), sub = lane / 16, sl = lane % 16;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t w = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; w < nw; w += waves) {   // uniform over the wave
        uint32_t open = ~visited[w];
        if (w == nw - 1 && (n & 31)) open &= (1u << (n & 31)) - 1u;
        // the wavefront's four lane groups share the word: group k takes its k-th, (k+4)-th, ... unreached vertex (a
        // vertex is a chain of dependent loads; four chains run side by side)
        uint32_t mine = 0u;
        for (int k = 0; open; ++k) {   // uniform over the wave
            const uint32_t lowest = open & (0u - open);
            open ^= lowest;
            if ((k & 3) == sub) mine |= lowest;
        }
        while (mine) {   // uniform over the lane group
            const int b = __ffs(mine) - 1;
            mine &= mine - 1u;
            const int32_t v = (int32_t)(w * 32 + b);
            const int32_t s = row_ptr_t[v], e = row_ptr_t[v + 1];
            if (e - s > kAsHubDegree) {
                if (sl == 0) hubq[atomicAdd(&ctrl->n_hubs, 1)] = v;
                continue;
            }
            bool found = false;
            for (int32_t p = s; p < e && !found; p += 64) {
                int32_t u[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) u[j] = p + j * 16 + sl < e ? col_idx_t[p + j * 16 + sl] : -1;
                bool hit = false;
#pragma unroll
                for (int j = 0; j < 4; ++j) hit |= u[j] >= 0 && in_set(frontier, u[j]);
                found = ((__ballot(hit) >> (sub * 16)) & 0xffffull) != 0ull;
            }
            if (found && sl == 0) seen[v] = 1;
        }
    }
}

// Long rows of a pull level: one workgroup per queued vertex, 256 entries per step, until one is in the frontier.
__global__ __launch_bounds__(256) void as_pull_hubs_kernel(const int32_t* __restrict__ row_ptr_t, const int32_t* __restrict__ col_idx_t,
                                                           uint8_t* __restrict__ seen, const uint32_t* __restrict__ frontier,
                                                           const int64_t* __restrict__ hop_offsets, int32_t ring, int32_t n,
                                                           int64_t nnz_t, const int32_t* __restrict__ hubq, const AsCtrl* ctrl) {
    if (!as_pull_level(ctrl, hop_offsets, ring, n, nnz_t)) return;
    const int32_t n_hubs = ctrl->n_hubs;
    for (int32_t h = blockIdx.x; h < n_hubs; h += gridDim.x) {   // uniform over the workgroup
        const int32_t v = hubq[h];
        const int32_t s = row_ptr_t[v], e = row_ptr_t[v + 1];
        for (int32_t base = s; base < e; base += 256) {
            const int32_t p = base + (int32_t)threadIdx.x;
            const int hit = p < e && in_set(frontier, col_idx_t[p]);
            if (__syncthreads_or(hit)) {
                if (threadIdx.x == 0) seen[v] = 1;
                break;
            }
        }
    }
}

__global__ __launch_bounds__(kAsWordsPerBlock) void as_count_kernel(const uint8_t* __restrict__ seen,
                                                                    const uint32_t* __restrict__ visited, int64_t nw,
                                                                    int32_t* __restrict__ blk_cnt) {
    __shared__ int s_part[kAsWordsPerBlock / kWave];
    const int64_t w = (int64_t)blockIdx.x * kAsWordsPerBlock + threadIdx.x;
    int c = 0;
    if (w < nw) c = __popc(as_mask_of_bytes(seen + 32 * w) & ~visited[w]);
    int total;
    block_exclusive_scan<kAsWordsPerBlock>(c, s_part, &total);
    if (threadIdx.x == 0) blk_cnt[blockIdx.x] = total;
}

__global__ __launch_bounds__(1024) void as_scan_kernel(int32_t* __restrict__ blk_cnt, int64_t n_blocks,
                                                       int64_t* __restrict__ hop_offsets, int32_t ring, AsCtrl* ctrl) {
    __shared__ int s_part[1024 / kWave];
    const int64_t total = single_block_exclusive_scan(blk_cnt, n_blocks, s_part);
    if (threadIdx.x == 0) {
        hop_offsets[ring + 1] = hop_offsets[ring] + total;
        ctrl->n_hubs = 0;
        ctrl->frontier_edges = 0ull;
    }
}

__global__ __launch_bounds__(kAsWordsPerBlock) void as_emit_kernel(const uint8_t* __restrict__ seen, uint32_t* __restrict__ visited,
                                                                   int64_t nw, const int32_t* __restrict__ blk_cnt,
                                                                   const int64_t* __restrict__ hop_offsets, int32_t ring,
                                                                   int32_t* __restrict__ ring_ids, int32_t* __restrict__ dist,
                                                                   uint32_t* __restrict__ frontier) {
    __shared__ int s_part[kAsWordsPerBlock / kWave];
    const int64_t w = (int64_t)blockIdx.x * kAsWordsPerBlock + threadIdx.x;
    uint32_t fresh = 0u;
    if (w < nw) {
        const uint32_t sn = as_mask_of_bytes(seen + 32 * w), vis = visited[w];
        fresh = sn & ~vis;
        if (fresh) visited[w] = vis | sn;
        if (frontier != nullptr) frontier[w] = fresh;   // the ring a pull level looks for
    }
    int total;
    const int before = block_exclusive_scan<kAsWordsPerBlock>(__popc(fresh), s_part, &total);
    int64_t pos = hop_offsets[ring] + blk_cnt[blockIdx.x] + before;
    while (fresh) {
        const int b = __ffs(fresh) - 1;
        fresh &= fresh - 1;
        const int32_t v = (int32_t)(w * 32 + b);
        ring_ids[pos++] = v;
        dist[v] = ring;
    }
}

// ---- expansion-aware traversal (paper section 5.3.1) -----------------------------------------------------------
// The same level-synchronous scheme with a thinned expansion: a traversed vertex keeps at most `fanout` of its
// not-yet-selected neighbours, those with the smallest (key, id).  `visited` is read-only while a hop expands, so
// "not yet selected" means "when the hop started" for every row, and the result does not depend on the order in
// which rows are processed.  Keys: the seeded edge hash of the boundary sampler, or (the paper's rule) the negated
// number of connections of the candidate to vertices that were unselected when the hop started.

// conn[u] = number of entries of row u that are not in `visited`; sixteen lanes per row
__global__ __launch_bounds__(256) void eas_connections_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                                                               int32_t n, const uint32_t* __restrict__ visited,
                                                               int32_t* __restrict__ conn) {
    const int lane = lane_id(), sub = lane / 16, sl = lane % 16;
    const int64_t groups = (int64_t)gridDim.x * (blockDim.x / 16);
    for (int64_t u = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / 16; u < n; u += groups) {
        const int32_t s = row_ptr[u], e = row_ptr[u + 1];
        int32_t c = 0;
        for (int32_t p = s; p < e; p += 16) {
            const bool open = p + sl < e && !in_set(visited, col_idx[p + sl]);
            c += __popcll((__ballot(open) >> (sub * 16)) & 0xffffull);
        }
        if (sl == 0) conn[u] = c;
    }
}

__device__ __forceinline__ uint64_t eas_key(int32_t rule, uint64_t seed_hop_mixed, const int32_t* __restrict__ conn, int32_t v, int32_t u) {
    return rule == 1 ? (uint64_t)(0xffffffffu - (uint32_t)conn[u]) : edge_key(seed_hop_mixed, (uint64_t)v, (uint64_t)u);
}

constexpr int kEasShortRow = 64;    // rows up to this length: sixteen lanes each; longer rows: a wavefront each
constexpr int kEasListCap = 1024;   // candidates of one long row that a wavefront keeps in LDS

// Rows of at most kEasShortRow entries: sixteen lanes per frontier vertex, four vertices per wavefront, up to four
// entries of the row per lane.  Entries, candidate flags and keys are read once and stay in registers; a row with
// more than `fanout` candidates finds the fanout-th smallest (key, id) by `fanout` rounds of "smallest pair above the
// previous one" over those registers.  Every lane runs every ballot and shuffle (no lane leaves early).
__global__ __launch_bounds__(256) void eas_expand_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                                                          const int32_t* __restrict__ ring_ids, const int64_t* __restrict__ hop_offsets,
                                                          int32_t ring, const uint32_t* __restrict__ visited, uint8_t* __restrict__ seen,
                                                          int32_t fanout, int32_t rule, uint64_t seed_hop_mixed,
                                                          const int32_t* __restrict__ conn) {
    constexpr int kPerLane = kEasShortRow / 16;
    const int64_t begin = hop_offsets[ring], end = hop_offsets[ring + 1];
    const int lane = lane_id(), sub = lane / 16, sl = lane % 16;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    if (fanout == 0) return;   // nothing is selected
    for (int64_t base = begin + 4 * (((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6); base < end; base += 4 * waves) {  // uniform over the wave
        const int64_t i = base + sub;
        int32_t v = 0, s = 0, e = 0;
        if (i < end) {
            v = ring_ids[i];
            s = row_ptr[v];
            e = row_ptr[v + 1];
            if (e - s > kEasShortRow) e = s;   // eas_expand_long_kernel takes this row
        }
        int32_t u[kPerLane];
        bool cand[kPerLane];
        uint64_t key[kPerLane];
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) u[j] = s + j * 16 + sl < e ? col_idx[s + j * 16 + sl] : -1;
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) cand[j] = u[j] >= 0 && !in_set(visited, u[j]);
        int32_t n_cand = 0;
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) {
            key[j] = cand[j] ? eas_key(rule, seed_hop_mixed, conn, v, u[j]) : ~0ull;
            n_cand += __popcll((__ballot(cand[j]) >> (sub * 16)) & 0xffffull);
        }
        // threshold pair: candidates with (key, id) <= (thr_k, thr_u) are kept
        uint64_t thr_k = ~0ull;
        int32_t thr_u = 0x7fffffff;
        const bool need = n_cand > fanout;   // uniform over the 16-lane group
        if (__ballot(need) != 0ull) {        // uniform over the wavefront
            uint64_t prev_k = 0ull;
            int32_t prev_u = -1;
            for (int32_t round = 0; round < fanout; ++round) {
                uint64_t best_k = ~0ull;
                int32_t best_u = 0x7fffffff;
#pragma unroll
                for (int j = 0; j < kPerLane; ++j) {
                    if (cand[j] && pair_less(prev_k, prev_u, key[j], u[j]) && pair_less(key[j], u[j], best_k, best_u)) {
                        best_k = key[j];
                        best_u = u[j];
                    }
                }
#pragma unroll
                for (int d = 8; d >= 1; d >>= 1) {
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
            if (cand[j] && !pair_less(thr_k, thr_u, key[j], u[j]) && !seen[u[j]]) seen[u[j]] = 1;
        }
    }
}

// Rows longer than kEasShortRow: one wavefront per frontier vertex.  The row is read ONCE; its candidates (neighbours
// not selected when the hop started) go to a list in LDS with their keys (one key computation and, for the
// best-connected-first rule, one read of conn[] per candidate).  When the list is full it is cut down to its `fanout`
// smallest (key, id) pairs, and from then on only candidates below the largest of those are listed: a pair that is
// not among the fanout smallest of what has been read so far cannot be among the fanout smallest of the row.  At the
// end the fanout smallest pairs of the list are the row's.  (A fanout too large for this - within 64 of the list's
// capacity - takes the rounds over the row itself, re-reading it once per kept neighbour.)
__global__ __launch_bounds__(256) void eas_expand_long_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                                                               const int32_t* __restrict__ ring_ids,
                                                               const int64_t* __restrict__ hop_offsets, int32_t ring,
                                                               const uint32_t* __restrict__ visited, uint8_t* __restrict__ seen,
                                                               int32_t fanout, int32_t rule, uint64_t seed_hop_mixed,
                                                               const int32_t* __restrict__ conn) {
    __shared__ uint64_t s_key[4][kEasListCap];
    __shared__ int32_t s_id[4][kEasListCap];
    const int64_t begin = hop_offsets[ring], end = hop_offsets[ring + 1];
    const int lane = lane_id(), wave = (int)(threadIdx.x >> 6);
    uint64_t* key = s_key[wave];
    int32_t* id = s_id[wave];
    const uint64_t lanes_below = (1ull << lane) - 1ull;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    if (fanout == 0) return;   // nothing is selected
    const bool streaming = fanout <= kEasListCap - kWave;   // the list can always be cut down far enough to take a chunk
    for (int64_t i = begin + (((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6); i < end; i += waves) {   // uniform over the wave
        const int32_t v = ring_ids[i];
        const int32_t s = row_ptr[v], e = row_ptr[v + 1];
        if (e - s <= kEasShortRow) continue;
        uint64_t thr_k = ~0ull;   // pairs above (thr_k, thr_u) are out
        int32_t thr_u = 0x7fffffff;
        int32_t n_list = 0;       // pairs in the list
        int32_t n_cand = 0;       // candidates of the row (only needed when not streaming)
        for (int32_t p = s; p < e; p += kWave) {
            const int32_t q = p + lane;
            const int32_t u = q < e ? col_idx[q] : 0;
            const bool cand = q < e && !in_set(visited, u);
            const uint64_t k = cand ? eas_key(rule, seed_hop_mixed, conn, v, u) : 0ull;
            bool take = cand && !pair_less(thr_k, thr_u, k, u);
            uint64_t mask = __ballot(take);
            n_cand += __popcll(__ballot(cand));
            if (streaming && n_list + __popcll(mask) > kEasListCap) {   // uniform: cut the list down to its fanout smallest
                wave_lds_sync();
                wave_list_kth(key, id, n_list, fanout, lane, thr_k, thr_u);
                n_list = wave_list_keep_below(key, id, n_list, thr_k, thr_u, lane);
                take = cand && !pair_less(thr_k, thr_u, k, u);
                mask = __ballot(take);
            }
            const int32_t pos = n_list + __popcll(mask & lanes_below);
            if (take && pos < kEasListCap) {
                key[pos] = k;
                id[pos] = u;
            }
            n_list += __popcll(mask);
        }
        wave_lds_sync();
        if (streaming || n_list <= kEasListCap) {
            if (n_list > fanout) wave_list_kth(key, id, n_list, fanout, lane, thr_k, thr_u);
            for (int32_t j = lane; j < n_list; j += kWave) {
                const int32_t u = id[j];
                if (!pair_less(thr_k, thr_u, key[j], u) && !seen[u]) seen[u] = 1;
            }
        } else {
            // more candidates than the list holds and a fanout too large to cut it down: rounds over the row itself
            if (n_cand > fanout) {
                uint64_t prev_k = 0ull;
                int32_t prev_u = -1;
                for (int32_t round = 0; round < fanout; ++round) {
                    uint64_t best_k = ~0ull;
                    int32_t best_u = 0x7fffffff;
                    for (int32_t p = s + lane; p < e; p += kWave) {
                        const int32_t u = col_idx[p];
                        if (in_set(visited, u)) continue;
                        const uint64_t k = eas_key(rule, seed_hop_mixed, conn, v, u);
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
            for (int32_t p = s + lane; p < e; p += kWave) {
                const int32_t u = col_idx[p];
                if (in_set(visited, u)) continue;
                if (!pair_less(thr_k, thr_u, eas_key(rule, seed_hop_mixed, conn, v, u), u) && !seen[u]) seen[u] = 1;
            }
        }
        wave_lds_sync();   // the lists are read before the next row overwrites them
    }
}

}  // namespace gnnhot

using namespace gnnhot;

extern "C" int32_t gnn_build_active_sets(const gnn_csr* g, const gnn_csr* gt, const int32_t* targets, int32_t n_targets, int32_t L,
                                         int32_t* dist, int32_t* ring_ids, int64_t* hop_offsets, int64_t* hop_offsets_host,
                                         void* ws, size_t* ws_bytes, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    GNN_CHECK(check_csr(g, "g"));
    GNN_REQUIRE(g->n_rows == g->n_cols, GNN_ERR_SHAPE, "active sets need a square graph (%d x %d)", g->n_rows, g->n_cols);
    if (gt != nullptr) {
        GNN_CHECK(check_csr(gt, "gt"));
        GNN_REQUIRE(gt->n_rows == g->n_rows && gt->n_cols == g->n_cols && gt->nnz == g->nnz, GNN_ERR_SHAPE,
                    "gt (%d x %d, %lld entries) is not the transpose of g (%d x %d, %lld entries)", gt->n_rows, gt->n_cols,
                    (long long)gt->nnz, g->n_rows, g->n_cols, (long long)g->nnz);
    }
    GNN_REQUIRE(L >= 1 && L <= 1024, GNN_ERR_INVALID_ARG, "L = %d out of range [1, 1024]", L);
    GNN_REQUIRE(n_targets >= 0, GNN_ERR_INVALID_ARG, "n_targets < 0");
    const int32_t n = g->n_rows;
    const int64_t nw = ((int64_t)n + 31) / 32;
    const int64_t nb = nw > 0 ? (nw + kAsWordsPerBlock - 1) / kAsWordsPerBlock : 1;

    WsCarver carve(ws);
    uint32_t* visited = carve.take<uint32_t>((size_t)nw + 1);
    uint8_t* seen = carve.take<uint8_t>((size_t)nw * 32 + 32);
    uint32_t* frontier = carve.take<uint32_t>((size_t)nw + 1);
    int32_t* blk_cnt = carve.take<int32_t>((size_t)nb + 1);
    int32_t* hubq = carve.take<int32_t>((size_t)n + 1);
    AsCtrl* ctrl = carve.take<AsCtrl>(1);
    bool query;
    GNN_CHECK(ws_protocol(ws, ws_bytes, carve.used, &query));
    if (query) return GNN_OK;

    GNN_REQUIRE(hop_offsets != nullptr, GNN_ERR_INVALID_ARG, "hop_offsets is NULL");
    GNN_REQUIRE(n == 0 || (dist != nullptr && ring_ids != nullptr), GNN_ERR_INVALID_ARG, "dist / ring_ids is NULL");
    GNN_REQUIRE(n_targets == 0 || targets != nullptr, GNN_ERR_INVALID_ARG, "targets is NULL");

    as_init_kernel<<<grid_for(n > L + 2 ? n : L + 2, 256, 2048), 256, 0, stream>>>(dist, n, visited, seen, nw, ctrl, hop_offsets, L);
    GNN_LAUNCH_CHECK("as_init_kernel");
    if (n > 0) {
        if (n_targets > 0) {
            as_seed_kernel<<<grid_for(n_targets, 256, 2048), 256, 0, stream>>>(targets, n_targets, n, seen);
            GNN_LAUNCH_CHECK("as_seed_kernel");
        }
        const int expand_grid = 2048;  // 8 waves per CU-slot; bounds are read on the device
        const int64_t nnz_t = gt != nullptr ? gt->nnz : -1;   // < 0: every level pushes
        for (int32_t ring = 0; ring <= L; ++ring) {
            if (ring > 0) {
                if (gt != nullptr) {
                    as_plan_kernel<<<512, 256, 0, stream>>>(g->row_ptr, gt->row_ptr, ring_ids, hop_offsets, ring - 1, ctrl);
                    GNN_LAUNCH_CHECK("as_plan_kernel");
                }
                as_expand_kernel<<<expand_grid, 256, 0, stream>>>(g->row_ptr, g->col_idx, ring_ids, hop_offsets, ring - 1, seen, hubq, ctrl,
                                                                  n, nnz_t);
                GNN_LAUNCH_CHECK("as_expand_kernel");
                as_expand_hubs_kernel<<<2048, 256, 0, stream>>>(g->row_ptr, g->col_idx, seen, hubq, ctrl);
                GNN_LAUNCH_CHECK("as_expand_hubs_kernel");
                if (gt != nullptr) {
                    as_pull_kernel<<<grid_for(nw * kWave, 256, 8192), 256, 0, stream>>>(gt->row_ptr, gt->col_idx, n, nw, visited, seen,
                                                                                           frontier, hop_offsets, ring - 1, nnz_t, hubq, ctrl);
                    GNN_LAUNCH_CHECK("as_pull_kernel");
                    as_pull_hubs_kernel<<<1024, 256, 0, stream>>>(gt->row_ptr, gt->col_idx, seen, frontier, hop_offsets, ring - 1, n, nnz_t,
                                                                  hubq, ctrl);
                    GNN_LAUNCH_CHECK("as_pull_hubs_kernel");
                }
            }
            as_count_kernel<<<(int)nb, kAsWordsPerBlock, 0, stream>>>(seen, visited, nw, blk_cnt);
            GNN_LAUNCH_CHECK("as_count_kernel");
            as_scan_kernel<<<1, 1024, 0, stream>>>(blk_cnt, nb, hop_offsets, ring, ctrl);
            GNN_LAUNCH_CHECK("as_scan_kernel");
            as_emit_kernel<<<(int)nb, kAsWordsPerBlock, 0, stream>>>(seen, visited, nw, blk_cnt, hop_offsets, ring, ring_ids, dist,
                                                                     gt != nullptr ? frontier : nullptr);
            GNN_LAUNCH_CHECK("as_emit_kernel");
        }
    }
    if (hop_offsets_host != nullptr) {
        GNN_HIP(hipMemcpyAsync(hop_offsets_host, hop_offsets, sizeof(int64_t) * (size_t)(L + 2), hipMemcpyDeviceToHost, stream));
        GNN_HIP(hipStreamSynchronize(stream));
    }
    return GNN_OK;
}

extern "C" int32_t gnn_eas_traverse(const gnn_csr* g, const int32_t* targets, int32_t n_targets, int32_t hops, int32_t fanout,
                                    int32_t rule, uint64_t seed, int32_t* dist, int32_t* ring_ids, int64_t* hop_offsets,
                                    int64_t* hop_offsets_host, void* ws, size_t* ws_bytes, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    GNN_CHECK(check_csr(g, "g"));
    GNN_REQUIRE(g->n_rows == g->n_cols, GNN_ERR_SHAPE, "the traversal needs a square graph (%d x %d)", g->n_rows, g->n_cols);
    GNN_REQUIRE(hops >= 1 && hops <= 1024, GNN_ERR_INVALID_ARG, "hops = %d out of range [1, 1024]", hops);
    GNN_REQUIRE(fanout >= 0, GNN_ERR_INVALID_ARG, "fanout < 0");
    GNN_REQUIRE(rule == GNN_EAS_HASH || rule == GNN_EAS_DEGREE, GNN_ERR_INVALID_ARG, "unknown selection rule %d", rule);
    GNN_REQUIRE(n_targets >= 0, GNN_ERR_INVALID_ARG, "n_targets < 0");
    const int32_t n = g->n_rows;
    const int64_t nw = ((int64_t)n + 31) / 32;
    const int64_t nb = nw > 0 ? (nw + kAsWordsPerBlock - 1) / kAsWordsPerBlock : 1;

    WsCarver carve(ws);
    uint32_t* visited = carve.take<uint32_t>((size_t)nw + 1);
    uint8_t* seen = carve.take<uint8_t>((size_t)nw * 32 + 32);
    int32_t* blk_cnt = carve.take<int32_t>((size_t)nb + 1);
    int32_t* conn = carve.take<int32_t>(rule == GNN_EAS_DEGREE ? (size_t)n + 1 : 1);
    AsCtrl* ctrl = carve.take<AsCtrl>(1);
    bool query;
    GNN_CHECK(ws_protocol(ws, ws_bytes, carve.used, &query));
    if (query) return GNN_OK;

    GNN_REQUIRE(hop_offsets != nullptr, GNN_ERR_INVALID_ARG, "hop_offsets is NULL");
    GNN_REQUIRE(n == 0 || (dist != nullptr && ring_ids != nullptr), GNN_ERR_INVALID_ARG, "dist / ring_ids is NULL");
    GNN_REQUIRE(n_targets == 0 || targets != nullptr, GNN_ERR_INVALID_ARG, "targets is NULL");

    as_init_kernel<<<grid_for(n > hops + 2 ? n : hops + 2, 256, 2048), 256, 0, stream>>>(dist, n, visited, seen, nw, ctrl, hop_offsets, hops);
    GNN_LAUNCH_CHECK("as_init_kernel");
    if (n > 0) {
        if (n_targets > 0) {
            as_seed_kernel<<<grid_for(n_targets, 256, 2048), 256, 0, stream>>>(targets, n_targets, n, seen);
            GNN_LAUNCH_CHECK("as_seed_kernel");
        }
        for (int32_t ring = 0; ring <= hops; ++ring) {
            if (ring > 0) {
                if (rule == GNN_EAS_DEGREE) {
                    eas_connections_kernel<<<grid_for((int64_t)n * 16, 256, 1 << 16), 256, 0, stream>>>(g->row_ptr, g->col_idx, n, visited, conn);
                    GNN_LAUNCH_CHECK("eas_connections_kernel");
                }
                eas_expand_kernel<<<2048, 256, 0, stream>>>(g->row_ptr, g->col_idx, ring_ids, hop_offsets, ring - 1, visited, seen, fanout,
                                                            rule, mix64(seed + (uint64_t)ring), conn);
                GNN_LAUNCH_CHECK("eas_expand_kernel");
                eas_expand_long_kernel<<<2048, 256, 0, stream>>>(g->row_ptr, g->col_idx, ring_ids, hop_offsets, ring - 1, visited, seen, fanout,
                                                                 rule, mix64(seed + (uint64_t)ring), conn);
                GNN_LAUNCH_CHECK("eas_expand_long_kernel");
            }
            as_count_kernel<<<(int)nb, kAsWordsPerBlock, 0, stream>>>(seen, visited, nw, blk_cnt);
            GNN_LAUNCH_CHECK("as_count_kernel");
            as_scan_kernel<<<1, 1024, 0, stream>>>(blk_cnt, nb, hop_offsets, ring, ctrl);
            GNN_LAUNCH_CHECK("as_scan_kernel");
            as_emit_kernel<<<(int)nb, kAsWordsPerBlock, 0, stream>>>(seen, visited, nw, blk_cnt, hop_offsets, ring, ring_ids, dist, nullptr);
            GNN_LAUNCH_CHECK("as_emit_kernel");
        }
    }
    if (hop_offsets_host != nullptr) {
        GNN_HIP(hipMemcpyAsync(hop_offsets_host, hop_offsets, sizeof(int64_t) * (size_t)(hops + 2), hipMemcpyDeviceToHost, stream));
        GNN_HIP(hipStreamSynchronize(stream));
    }
    return GNN_OK;
}
