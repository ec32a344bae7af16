// Masked CSR aggregation, forward and backward (paper section 2.1: h_N(v) = AGGREGATE of the
// neighbours' hidden vectors, a scaled sum; section 6: only the rows the layer's mask keeps).
//
//     Y[v, :] = out_scale[v] * sum_{u in row(v), keep(u)} nbr_scale[u] * X[u, :]      v in rows
//
// Forward: (out_scale, nbr_scale) = (row_scale, col_scale), no filter.  Backward runs the
// same gather over the transposed graph with the scale roles swapped and keep(u) =
// "u was an active row of the forward call" (a dist probe), so no floating-point atomics
// are needed and results are bit-reproducible.
//
// Mapping to CDNA4.  The work is a gather of whole feature rows: HBM/L2 bound, one FMA per
// loaded element, so no MFMA.  A group of LPR lanes (16, 32 or 64) owns one output row and
// spans its feature columns with 16-byte loads, so every neighbour costs one fully coalesced
// row read; 64/LPR rows share a wavefront when rows are narrow.  Neighbour ids are fetched one
// tile ahead, coalesced, filtered, compacted and staged in an LDS tile private to the
// wavefront; the inner loop then reads the tile by broadcast and keeps U x NCH independent
// 16-byte loads in flight per lane.  Groups claim rows dynamically inside a workgroup's chunk.  Rows of more than kHubTiles tiles
// (power-law hubs) are split over all wavefronts of the workgroup and the partial sums are
// reduced through LDS in a fixed order, inside the same launch.
#include "common.h"
#include "scan.h"
#include <mutex>

namespace gnnhot {

// Independent row loads in flight per lane (a round), and workgroups per CU, when a lane owns one 16-byte chunk of
// the row.  A round must divide the tile (16, 32 or 64 entries): 6, 10 or 12 loads were all slower than 8.  Measured
// as the step time of the 8-level bf16 workload / the sampled-partition workload (ms; rows of 256 and 512 bytes, 10
// to 20 neighbours, partitions numbered by (distance, id)): rounds of 16 at 4 workgroups per CU 17.5 / 23.7, 8 at 6
// 17.5 / 24.2, 8 at 5 or 4 16.5 / 23.4, 4 at 8 19.5 / 24.8 - slots of a round past the end of a tile are wasted issue
// slots of the vector cache, but eight workgroups of short rounds lose more to the caches than they gain.  (On the
// same graph numbered by global id the order is the reverse, 4 at 8 being 18 % faster than 16 at 4: the setting
// follows the numbering the extraction produces.)  Rows of 1 KB (64 lanes per row): 8 at 5 (8 at 6: +2 %).
#ifndef GNN_SPMM_U_NARROW
#define GNN_SPMM_U_NARROW 8
#endif
#ifndef GNN_SPMM_U_WIDE
#define GNN_SPMM_U_WIDE 8
#endif
#ifndef GNN_SPMM_MINB_NARROW
#define GNN_SPMM_MINB_NARROW 5
#endif
#ifndef GNN_SPMM_MINB_WIDE
#define GNN_SPMM_MINB_WIDE 5
#endif

// Rows of the list per lane group in one workgroup, and the length (in tiles of LPR entries) from which a row is
// split over all groups of the workgroup.  A group walks a row alone, tile by tile; with power-law rows one long row
// keeps its group - and the workgroup's registers and LDS - busy long after the other groups have run out of rows
// (simulated on the 8-level workload's graph: the groups of a 64-row workgroup are busy 35 % of its lifetime when only
// rows above 1024 entries are split).  Small chunks let the hardware's workgroup dispatch do the balancing, and a low
// split length bounds what one group can be left with.  Measured as the step time of the 8-level / the
// sampled-partition workload (ms): 4 rows per group and rows split above 1024 entries 16.5 / 23.4; 4 and 16 tiles
// 15.9 / 22.6; 2 and 16 tiles 15.2 / 21.4; 2 and 4 tiles 14.1 / 20.7; 3 and 4..12 tiles 14.0 / 21.4; 1 row per group
// 17.4 / 22.5; 8 or 16 rows per group 21.6 .. 31 / 24.4 .. 28.
#ifndef GNN_SPMM_RPG
#define GNN_SPMM_RPG 2
#endif
constexpr int kRowsPerGroup = GNN_SPMM_RPG;   // largest chunk: this many rows of the list per group
#ifndef GNN_SPMM_HUB_TILES
#define GNN_SPMM_HUB_TILES 4
#endif
constexpr int kHubTiles = GNN_SPMM_HUB_TILES;   // rows of more tiles (of LPR entries) than this are split over the whole workgroup
constexpr int kMaxChunk = 256;                  // rows of the list per workgroup, at most (one descriptor per thread)

// Column-blocked route (dense graphs, gathered matrix far larger than an L2).  The neighbour-id
// range [0, n_cols) is cut into 8 * passes equal blocks; in pass p workgroup i gathers, for its
// rows, only the neighbours inside block 8p + (i mod 8).  Workgroups are dealt round-robin to the 8
// compute dies, so every die's L2 sees one eighth of the matrix - and with the feature axis walked
// in slabs of 256 bytes per row (grid.y, the slow grid axis) that eighth fits: the gathers then
// run at L2 rather than at fabric speed (measured about 2x).  Each die leaves a plane of float
// partial sums; a second kernel adds the planes in block order and applies the output scale.
constexpr int kDies = 8;
#ifndef GNN_SPMM_DIE_BYTES
#define GNN_SPMM_DIE_BYTES (8ll << 20)      // target size of one die's share of one slab
#endif
#ifndef GNN_SPMM_BLOCKED_MIN_SLAB
#define GNN_SPMM_BLOCKED_MIN_SLAB (16ll << 20)   // below this slab size the plain route is already cache-resident
#endif
#ifndef GNN_SPMM_BLOCKED_MIN_SEG
#define GNN_SPMM_BLOCKED_MIN_SEG 8          // average neighbours of a row inside one column block
#endif
constexpr int kSlabBytes = 256;

struct SpmmArgs {
    const int32_t* row_ptr;
    const int32_t* col_idx;
    const int32_t* rows;      // nullable
    int32_t n_active;
    const void* X;
    int64_t ldx;
    void* Y;
    int64_t ldy;
    int32_t F;
    const float* out_scale;   // nullable, indexed by output row
    const float* nbr_scale;   // nullable, indexed by neighbour
    const int32_t* dist;      // nullable filter: keep u iff 0 <= dist[u] <= max_dist
    int32_t max_dist;
    const uint32_t* edge_keep;  // nullable filter: keep the entry at position p iff bit p is set (layer-wise sampling mask)
    int32_t cut_id;           // -1, or (rows sorted by column): every row ends at its first entry >= cut_id
    int32_t id_limit;         // -1, or (rows in any order): the filter drops the entries >= id_limit
    int32_t accumulate;
    const void* relu_h;       // nullable: the stored result is zeroed where this matrix (same rows and columns as Y) is <= 0
    int64_t ldh;
    int32_t rows_per_group;   // 1..kRowsPerGroup: rows of the list per LPR-lane group in one workgroup
    uint32_t x_row_bytes;     // > 0: X holds fewer than 2^24 rows and less than 4 GB, a row starts every x_row_bytes bytes - the
                              // row kernel then forms a gather address with one 24-bit multiply-add instead of a 64-bit product
    // column-blocked route only
    const int32_t* seg;       // [n_active][n_blocks + 1] cut points of every listed row: block j = [seg[j], seg[j+1])
    const int32_t* seg_end;   // nullable, [n_active][n_blocks]: block j ends here instead (filtered, compacted copy of the ids)
    const float* edge_w;      // with a neighbour scale: the factor of every entry of col_idx, at the same position
    int32_t n_blocks;
    int32_t block0;           // first column block of this pass
};

// ---- element access: VE elements per lane-chunk ------------------------------------------
template <int DT, int VE>
struct Elem;

template <>
struct Elem<GNN_F32, 4> {
    static constexpr int VE = 4;
    using Raw = uint4;
    static __device__ __forceinline__ Raw load(const void* p, int64_t off) { return *(const uint4*)((const float*)p + off); }
    static __device__ __forceinline__ void fma(float (&acc)[4], float w, const Raw& r) {
        acc[0] = fmaf(w, __uint_as_float(r.x), acc[0]);
        acc[1] = fmaf(w, __uint_as_float(r.y), acc[1]);
        acc[2] = fmaf(w, __uint_as_float(r.z), acc[2]);
        acc[3] = fmaf(w, __uint_as_float(r.w), acc[3]);
    }
    // h (nullable): activation matrix of the same layout position hoff; what is stored is zeroed where h <= 0.
    // h == p stands for "the value being stored itself": the store applies a ReLU.
    static __device__ __forceinline__ void store(void* p, int64_t off, const float (&v)[4], int n_valid, bool accumulate,
                                                 const void* h = nullptr, int64_t hoff = 0) {
        float* q = (float*)p + off;
        const float* hq = (const float*)h + hoff;
        if (n_valid >= 4) {
            float4 o = make_float4(v[0], v[1], v[2], v[3]);
            if (accumulate) {
                float4 old = *(const float4*)q;
                o.x += old.x; o.y += old.y; o.z += old.z; o.w += old.w;
            }
            if (h) {
                const float4 m = h == p ? o : *(const float4*)hq;
                o.x = m.x > 0.f ? o.x : 0.f; o.y = m.y > 0.f ? o.y : 0.f; o.z = m.z > 0.f ? o.z : 0.f; o.w = m.w > 0.f ? o.w : 0.f;
            }
            *(float4*)q = o;
        } else {
            for (int e = 0; e < n_valid; ++e) {
                const float t = accumulate ? q[e] + v[e] : v[e];
                q[e] = (h == nullptr || (h == p ? t : hq[e]) > 0.f) ? t : 0.f;
            }
        }
    }
};

template <>
struct Elem<GNN_F32, 1> {
    static constexpr int VE = 1;
    using Raw = float;
    static __device__ __forceinline__ Raw load(const void* p, int64_t off) { return ((const float*)p)[off]; }
    static __device__ __forceinline__ float to_float(Raw r) { return r; }
    static __device__ __forceinline__ void fma(float (&acc)[1], float w, const Raw& r) { acc[0] = fmaf(w, r, acc[0]); }
    static __device__ __forceinline__ void store(void* p, int64_t off, const float (&v)[1], int n_valid, bool accumulate,
                                                 const void* h = nullptr, int64_t hoff = 0) {
        float* q = (float*)p + off;
        if (n_valid >= 1) {
            const float t = accumulate ? q[0] + v[0] : v[0];
            q[0] = (h == nullptr || (h == p ? t : ((const float*)h)[hoff]) > 0.f) ? t : 0.f;
        }
    }
};

template <>
struct Elem<GNN_BF16, 8> {
    static constexpr int VE = 8;
    using Raw = uint4;
    static __device__ __forceinline__ Raw load(const void* p, int64_t off) { return *(const uint4*)((const uint16_t*)p + off); }
    static __device__ __forceinline__ void fma(float (&acc)[8], float w, const Raw& r) {
        acc[0] = fmaf(w, bf16lo(r.x), acc[0]); acc[1] = fmaf(w, bf16hi(r.x), acc[1]);
        acc[2] = fmaf(w, bf16lo(r.y), acc[2]); acc[3] = fmaf(w, bf16hi(r.y), acc[3]);
        acc[4] = fmaf(w, bf16lo(r.z), acc[4]); acc[5] = fmaf(w, bf16hi(r.z), acc[5]);
        acc[6] = fmaf(w, bf16lo(r.w), acc[6]); acc[7] = fmaf(w, bf16hi(r.w), acc[7]);
    }
    static __device__ __forceinline__ void store(void* p, int64_t off, const float (&v)[8], int n_valid, bool accumulate,
                                                 const void* h = nullptr, int64_t hoff = 0) {
        uint16_t* q = (uint16_t*)p + off;
        const uint16_t* hq = (const uint16_t*)h + hoff;
        if (n_valid >= 8) {
            float t[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) t[e] = v[e];
            if (accumulate) {
                uint4 old = *(const uint4*)q;
                t[0] += bf16lo(old.x); t[1] += bf16hi(old.x); t[2] += bf16lo(old.y); t[3] += bf16hi(old.y);
                t[4] += bf16lo(old.z); t[5] += bf16hi(old.z); t[6] += bf16lo(old.w); t[7] += bf16hi(old.w);
            }
            if (h == p) {
#pragma unroll
                for (int e = 0; e < 8; ++e) t[e] = t[e] > 0.f ? t[e] : 0.f;
            } else if (h) {
                const uint4 m = *(const uint4*)hq;
                t[0] = bf16lo(m.x) > 0.f ? t[0] : 0.f; t[1] = bf16hi(m.x) > 0.f ? t[1] : 0.f;
                t[2] = bf16lo(m.y) > 0.f ? t[2] : 0.f; t[3] = bf16hi(m.y) > 0.f ? t[3] : 0.f;
                t[4] = bf16lo(m.z) > 0.f ? t[4] : 0.f; t[5] = bf16hi(m.z) > 0.f ? t[5] : 0.f;
                t[6] = bf16lo(m.w) > 0.f ? t[6] : 0.f; t[7] = bf16hi(m.w) > 0.f ? t[7] : 0.f;
            }
            uint4 o;
            o.x = pack_bf16(t[0], t[1]); o.y = pack_bf16(t[2], t[3]);
            o.z = pack_bf16(t[4], t[5]); o.w = pack_bf16(t[6], t[7]);
            *(uint4*)q = o;
        } else {
            for (int e = 0; e < n_valid; ++e) {
                const float t = accumulate ? bf16_to_f32(q[e]) + v[e] : v[e];
                q[e] = f32_to_bf16((h == nullptr || (h == p ? t : bf16_to_f32(hq[e])) > 0.f) ? t : 0.f);
            }
        }
    }
};

// two bf16 per lane: narrow rows (up to 32 columns) spread over 16 lanes, so that a tile still holds 16 neighbours
template <>
struct Elem<GNN_BF16, 2> {
    static constexpr int VE = 2;
    using Raw = uint32_t;
    static __device__ __forceinline__ Raw load(const void* p, int64_t off) { return *(const uint32_t*)((const uint16_t*)p + off); }
    static __device__ __forceinline__ void fma(float (&acc)[2], float w, const Raw& r) {
        acc[0] = fmaf(w, bf16lo(r), acc[0]);
        acc[1] = fmaf(w, bf16hi(r), acc[1]);
    }
    static __device__ __forceinline__ void store(void* p, int64_t off, const float (&v)[2], int n_valid, bool accumulate,
                                                 const void* h = nullptr, int64_t hoff = 0) {
        uint16_t* q = (uint16_t*)p + off;
        const uint16_t* hq = (const uint16_t*)h + hoff;
        for (int e = 0; e < 2; ++e) {
            if (e >= n_valid) break;
            const float t = accumulate ? bf16_to_f32(q[e]) + v[e] : v[e];
            q[e] = f32_to_bf16((h == nullptr || (h == p ? t : bf16_to_f32(hq[e])) > 0.f) ? t : 0.f);
        }
    }
};

// four bf16 per lane (33 to 64 columns over 16 lanes)
template <>
struct Elem<GNN_BF16, 4> {
    static constexpr int VE = 4;
    using Raw = uint2;
    static __device__ __forceinline__ Raw load(const void* p, int64_t off) { return *(const uint2*)((const uint16_t*)p + off); }
    static __device__ __forceinline__ void fma(float (&acc)[4], float w, const Raw& r) {
        acc[0] = fmaf(w, bf16lo(r.x), acc[0]);
        acc[1] = fmaf(w, bf16hi(r.x), acc[1]);
        acc[2] = fmaf(w, bf16lo(r.y), acc[2]);
        acc[3] = fmaf(w, bf16hi(r.y), acc[3]);
    }
    static __device__ __forceinline__ void store(void* p, int64_t off, const float (&v)[4], int n_valid, bool accumulate,
                                                 const void* h = nullptr, int64_t hoff = 0) {
        uint16_t* q = (uint16_t*)p + off;
        const uint16_t* hq = (const uint16_t*)h + hoff;
        for (int e = 0; e < 4; ++e) {
            if (e >= n_valid) break;
            const float t = accumulate ? bf16_to_f32(q[e]) + v[e] : v[e];
            q[e] = f32_to_bf16((h == nullptr || (h == p ? t : bf16_to_f32(hq[e])) > 0.f) ? t : 0.f);
        }
    }
};

// two floats per lane (17 to 32 columns over 16 lanes)
template <>
struct Elem<GNN_F32, 2> {
    static constexpr int VE = 2;
    using Raw = float2;
    static __device__ __forceinline__ Raw load(const void* p, int64_t off) { return *(const float2*)((const float*)p + off); }
    static __device__ __forceinline__ void fma(float (&acc)[2], float w, const Raw& r) {
        acc[0] = fmaf(w, r.x, acc[0]);
        acc[1] = fmaf(w, r.y, acc[1]);
    }
    static __device__ __forceinline__ void store(void* p, int64_t off, const float (&v)[2], int n_valid, bool accumulate,
                                                 const void* h = nullptr, int64_t hoff = 0) {
        float* q = (float*)p + off;
        const float* hq = (const float*)h + hoff;
        for (int e = 0; e < 2; ++e) {
            if (e >= n_valid) break;
            const float t = accumulate ? q[e] + v[e] : v[e];
            q[e] = (h == nullptr || (h == p ? t : hq[e]) > 0.f) ? t : 0.f;
        }
    }
};

template <>
struct Elem<GNN_BF16, 1> {
    static constexpr int VE = 1;
    using Raw = uint16_t;
    static __device__ __forceinline__ Raw load(const void* p, int64_t off) { return ((const uint16_t*)p)[off]; }
    static __device__ __forceinline__ float to_float(Raw r) { return bf16_to_f32(r); }
    static __device__ __forceinline__ void fma(float (&acc)[1], float w, const Raw& r) { acc[0] = fmaf(w, bf16_to_f32(r), acc[0]); }
    static __device__ __forceinline__ void store(void* p, int64_t off, const float (&v)[1], int n_valid, bool accumulate,
                                                 const void* h = nullptr, int64_t hoff = 0) {
        uint16_t* q = (uint16_t*)p + off;
        if (n_valid >= 1) {
            const float t = accumulate ? bf16_to_f32(q[0]) + v[0] : v[0];
            q[0] = f32_to_bf16((h == nullptr || (h == p ? t : bf16_to_f32(((const uint16_t*)h)[hoff])) > 0.f) ? t : 0.f);
        }
    }
};

// Float partial sums of the column-blocked route: VE consecutive floats at p[off] (16-byte aligned when VE >= 4).
template <int VE>
__device__ __forceinline__ void store_part(float* p, int64_t off, const float (&v)[VE], int n_valid, bool accumulate) {
    if (VE >= 4 && n_valid == VE) {
#pragma unroll
        for (int q = 0; q < VE / 4; ++q) {
            float4* dst = (float4*)(p + off) + q;
            float4 o = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
            if (accumulate) {
                const float4 old = *dst;
                o.x += old.x; o.y += old.y; o.z += old.z; o.w += old.w;
            }
            *dst = o;
        }
    } else {
        for (int k = 0; k < n_valid; ++k) p[off + k] = accumulate ? p[off + k] + v[k] : v[k];
    }
}

// The value the filter tests for the entry at position p with neighbour u: dist[u] (0 without a dist filter),
// or -1 if the layer's edge mask drops the entry.
__device__ __forceinline__ int32_t filter_probe(const SpmmArgs& a, int32_t u, int32_t p) {
    int32_t d = a.dist ? a.dist[u] : 0;
    if (a.edge_keep && !((a.edge_keep[p >> 5] >> (p & 31)) & 1u)) d = -1;
    if (a.id_limit >= 0 && u >= a.id_limit) d = -1;
    return d;
}

// First position in [lo, hi) of a row sorted by column whose entry is >= bound (hi if none).
__device__ __forceinline__ int32_t row_lower_bound(const int32_t* __restrict__ col_idx, int32_t lo, int32_t hi, int64_t bound) {
    while (lo < hi) {
        const int32_t mid = lo + ((hi - lo) >> 1);
        if ((int64_t)col_idx[mid] < bound) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

// Filter (backward: "was u an active row of the forward call"), compact and stage one tile of
// neighbour ids (already in registers: `u` and its `d` = dist[u], valid where `in_row`) into the group's LDS slots.
// Returns how many were kept.
template <int LPR, bool FILTER>
__device__ __forceinline__ int commit_tile(const SpmmArgs& a, bool in_row, int32_t u, int32_t d, int n_in_row, int sub, int sl,
                                           int32_t* s_idx) {
    if (!FILTER) {
        if (in_row) s_idx[sub * LPR + sl] = u;
        return n_in_row;
    }
    const bool keep = in_row && d >= 0 && d <= a.max_dist;  // d = dist[u], fetched by the caller
    const uint64_t group_mask = LPR == 64 ? ~0ull : (((1ull << (LPR & 63)) - 1ull) << (sub * LPR));
    const uint64_t kept = __ballot(keep) & group_mask;
    const uint64_t below = kept & ((1ull << (sub * LPR + sl)) - 1ull);
    if (keep) s_idx[sub * LPR + __popcll(below)] = u;
    return __popcll(kept);
}

// acc += sum over the staged tile.  `cnt` (this group's entries) may differ between the groups
// of a wave; `cnt_max` is uniform over the wave.  Each round issues U x NCH independent row loads
// (plus U broadcast loads of the neighbour scale) before the first multiply-add.  The issue part has
// no branch that depends on a lane: a slot past the group's count repeats the group's last entry (a
// cache hit) and a lane past the row's width reads the row's start; only the multiply-adds are
// predicated.  (With a branch around every load the compiler put a wait for the id's LDS read and
// two mask updates between any two loads: sixteen loads took longer to issue than to arrive.)
template <typename E, int LPR, int NCH, int U>
__device__ __forceinline__ void consume_tile(const SpmmArgs& a, int cnt, int cnt_max, int sub, const int64_t (&col_off)[NCH],
                                             const bool (&col_ok)[NCH], const int32_t* s_idx, float (&acc)[NCH][E::VE]) {
    int64_t col_ld[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) col_ld[c] = col_ok[c] ? col_off[c] : 0;
    uint32_t col_ld_bytes[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) col_ld_bytes[c] = (uint32_t)col_ld[c] * (uint32_t)(sizeof(typename E::Raw) / E::VE);
    const int last = cnt > 0 ? cnt - 1 : 0;
    for (int k = 0; k < cnt_max; k += U) {
        typename E::Raw x[U][NCH];
        float w[U];
        int32_t u[U];
#pragma unroll
        for (int j = 0; j < U; ++j) {
            const int32_t staged = s_idx[sub * LPR + (k + j < cnt ? k + j : last)];
            u[j] = cnt > 0 ? staged : 0;   // nothing staged for this group: the slot may hold anything, row 0 always exists
        }
        if (a.nbr_scale) {   // uniform
#pragma unroll
            for (int j = 0; j < U; ++j) w[j] = a.nbr_scale[u[j]];
        } else {
#pragma unroll
            for (int j = 0; j < U; ++j) w[j] = 1.f;
        }
        if (a.x_row_bytes) {   // uniform
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const uint32_t base = __umul24((uint32_t)u[j], a.x_row_bytes);
#pragma unroll
                for (int c = 0; c < NCH; ++c) x[j][c] = *(const typename E::Raw*)((const char*)a.X + (base + col_ld_bytes[c]));
            }
        } else {
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const int64_t base = (int64_t)u[j] * a.ldx;
#pragma unroll
                for (int c = 0; c < NCH; ++c) x[j][c] = E::load(a.X, base + col_ld[c]);
            }
        }
#pragma unroll
        for (int j = 0; j < U; ++j) {
            if (k + j < cnt) {
#pragma unroll
                for (int c = 0; c < NCH; ++c)
                    if (col_ok[c]) E::fma(acc[c], w[j], x[j][c]);
            }
        }
    }
}


// One workgroup (4 wavefronts = NG groups of LPR lanes) owns NG * kRowsPerGroup consecutive
// entries of the row list.
//   phase 0  the row descriptors (id, start, end, output scale) of the chunk go to LDS in one
//            coalesced sweep;
//   phase 1  every group streams through rows of the chunk, one LPR-wide tile of neighbours per
//            step; a group that finishes a row claims the next unclaimed one from an LDS counter,
//            so short and long rows mix without idle groups, and the ids of the NEXT tile are
//            fetched while the current tile's rows are being gathered;
//   phase 2  hub rows (more than kHubTiles tiles) are taken one at a time by ALL groups (group q takes
//            tiles q, q+NG, ...); the partial sums meet in LDS and are added in group order.
// Which group handles a row does not change the order of its additions: results are bit-reproducible.
// Workgroups per CU: see the tuning constants at the head of the file.
template <int DT, int VE, int LPR, int NCH, int U, bool FILTER>
__global__ __launch_bounds__(256, NCH == 1 ? (LPR == 64 ? GNN_SPMM_MINB_WIDE : GNN_SPMM_MINB_NARROW) : 4) void spmm_rows_kernel(SpmmArgs a) {
    using E = Elem<DT, VE>;
    constexpr int RPW = kWave / LPR;
    constexpr int NG = 4 * RPW;
    constexpr int RPB = NG * kRowsPerGroup < kMaxChunk ? NG * kRowsPerGroup : kMaxChunk;  // largest chunk
    constexpr int W = LPR * NCH * VE;        // feature columns per workgroup (grid.y blocks cover F)
    __shared__ int32_t s_idx_all[4][kWave];
    __shared__ int32_t s_row_v[RPB], s_row_s[RPB], s_row_e[RPB], s_row_hub[RPB], s_row_he[RPB];
    __shared__ float s_row_sc[RPB];
    __shared__ int32_t s_next;
    __shared__ float s_red[NG][W];
    const int lane = lane_id(), wave = (int)(threadIdx.x >> 6);
    const int sub = lane / LPR, sl = lane % LPR;
    const int gi = wave * RPW + sub;
    int32_t* s_idx = s_idx_all[wave];

    // ---- phase 0
    const int rpb = NG * a.rows_per_group;
    const int64_t chunk0 = (int64_t)blockIdx.x * rpb;
    const int n_chunk = (int)(((int64_t)a.n_active - chunk0) < rpb ? ((int64_t)a.n_active - chunk0) : rpb);
    if ((int)threadIdx.x < n_chunk) {
        const int r = threadIdx.x;
        const int32_t v = a.rows ? a.rows[chunk0 + r] : (int32_t)(chunk0 + r);
        const int32_t s = a.row_ptr[v];
        int32_t e = a.row_ptr[v + 1];
        if (a.cut_id >= 0) e = row_lower_bound(a.col_idx, s, e, a.cut_id);   // the entries past it can never pass the filter
        const bool hub = e - s > kHubTiles * LPR;
        s_row_v[r] = v;
        s_row_s[r] = s;
        s_row_e[r] = hub ? s : e;
        s_row_he[r] = e;
        s_row_hub[r] = hub ? 1 : 0;
        s_row_sc[r] = a.out_scale ? a.out_scale[v] : 1.f;
    }
    if (threadIdx.x == 0) s_next = NG;
    __syncthreads();

    int64_t col_off[NCH];
    bool col_ok[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        col_off[c] = (int64_t)blockIdx.y * W + (int64_t)(sl + c * LPR) * VE;
        col_ok[c] = col_off[c] < a.F;
    }
    float acc[NCH][VE];
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int k = 0; k < VE; ++k) acc[c][k] = 0.f;

    // ---- phase 1
    // Tile descriptors (row slot j, position p, row end e, valid flag) of the current tile and of the
    // two tiles after it: ids are fetched two tiles ahead and their dist values (backward filter) one
    // tile ahead, so neither latency is paid between two gathers.
    auto advance = [&](int j, int32_t p, int32_t e, bool hv, int& jo, int32_t& po, int32_t& eo, bool& ho) {
        const bool done = hv && p + LPR >= e;
        int got = 0;
        if (done && sl == 0) got = atomicAdd(&s_next, 1);
        got = __shfl(got, sub * LPR, kWave);  // executed by every lane of the wave
        jo = j; po = p + LPR; eo = e; ho = hv;
        if (done) {
            jo = got;
            ho = jo < n_chunk;
            po = ho ? s_row_s[jo] : 0;
            eo = ho ? s_row_e[jo] : 0;
        }
    };
    int jc = gi;
    bool have = jc < n_chunk;
    int32_t pc = 0, ec = 0;
    if (have) {
        pc = s_row_s[jc];
        ec = s_row_e[jc];
    }
    int jn;
    int32_t pn, en;
    bool have_n;
    advance(jc, pc, ec, have, jn, pn, en, have_n);
    int32_t u_c = (have && pc + sl < ec) ? a.col_idx[pc + sl] : 0;
    int32_t u_n = (have_n && pn + sl < en) ? a.col_idx[pn + sl] : 0;
    int32_t d_c = 0;
    if (FILTER) d_c = (have && pc + sl < ec) ? filter_probe(a, u_c, pc + sl) : -1;
    while (__ballot(have) != 0ull) {  // uniform over the wave
        const bool row_done = have && pc + LPR >= ec;
        int jnn;
        int32_t pnn, enn;
        bool have_nn;
        advance(jn, pn, en, have_n, jnn, pnn, enn, have_nn);
        const int32_t u_nn = (have_nn && pnn + sl < enn) ? a.col_idx[pnn + sl] : 0;  // two tiles ahead
        int32_t d_n = 0;
        if (FILTER) d_n = (have_n && pn + sl < en) ? filter_probe(a, u_n, pn + sl) : -1;  // one tile ahead

        int left = have ? ec - pc : 0;
        left = left < 0 ? 0 : (left < LPR ? left : LPR);
        wave_lds_sync();  // the previous tile has been consumed
        const int cnt = commit_tile<LPR, FILTER>(a, sl < left, u_c, d_c, left, sub, sl, s_idx);
        int cnt_max = cnt;
#pragma unroll
        for (int d = LPR; d < kWave; d <<= 1) cnt_max = max(cnt_max, __shfl_xor(cnt_max, d, kWave));
        wave_lds_sync();
        consume_tile<E, LPR, NCH, U>(a, cnt, cnt_max, sub, col_off, col_ok, s_idx, acc);

        if (row_done) {
            if (!s_row_hub[jc]) {
                const int32_t v = s_row_v[jc];
                const float sc = s_row_sc[jc];
#pragma unroll
                for (int c = 0; c < NCH; ++c) {
                    if (col_ok[c]) {
                        float o[VE];
#pragma unroll
                        for (int k = 0; k < VE; ++k) o[k] = acc[c][k] * sc;
                        const int64_t rest = (int64_t)a.F - col_off[c];
                        E::store(a.Y, (int64_t)v * a.ldy + col_off[c], o, rest >= VE ? VE : (int)rest, a.accumulate != 0, a.relu_h,
                                 (int64_t)v * a.ldh + col_off[c]);
                    }
                }
            }
#pragma unroll
            for (int c = 0; c < NCH; ++c)
#pragma unroll
                for (int k = 0; k < VE; ++k) acc[c][k] = 0.f;
        }
        jc = jn; pc = pn; ec = en; have = have_n;
        jn = jnn; pn = pnn; en = enn; have_n = have_nn;
        u_c = u_n; u_n = u_nn; d_c = d_n;
    }

    // ---- phase 2
    __syncthreads();
    for (int q = 0; q < n_chunk; ++q) {
        if (!s_row_hub[q]) continue;  // uniform over the workgroup
        const int32_t hv = s_row_v[q];
        const int32_t hs = s_row_s[q], he = s_row_he[q];
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int k = 0; k < VE; ++k) acc[c][k] = 0.f;
        for (int64_t base = (int64_t)hs + (int64_t)wave * kWave; base < he; base += 4 * kWave) {
            // the wave's RPW groups take consecutive LPR-wide tiles of this 64-entry stretch
            const int64_t p0 = base + sub * LPR;
            int left = (int)((int64_t)he - p0 < 0 ? 0 : ((int64_t)he - p0 < LPR ? (int64_t)he - p0 : LPR));
            const int32_t u = sl < left ? a.col_idx[p0 + sl] : 0;
            int32_t d = 0;
            if (FILTER) d = sl < left ? filter_probe(a, u, (int32_t)(p0 + sl)) : -1;
            wave_lds_sync();
            const int cnt = commit_tile<LPR, FILTER>(a, sl < left, u, d, left, sub, sl, s_idx);
            int cnt_max = cnt;
#pragma unroll
            for (int d = LPR; d < kWave; d <<= 1) cnt_max = max(cnt_max, __shfl_xor(cnt_max, d, kWave));
            wave_lds_sync();
            consume_tile<E, LPR, NCH, U>(a, cnt, cnt_max, sub, col_off, col_ok, s_idx, acc);
        }
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int k = 0; k < VE; ++k) s_red[gi][(sl + c * LPR) * VE + k] = acc[c][k];
        __syncthreads();
        const float sc = s_row_sc[q];
        for (int col = threadIdx.x; col < W; col += 256) {
            const int64_t gcol = (int64_t)blockIdx.y * W + col;
            if (gcol < a.F) {
                float t = 0.f;
#pragma unroll
                for (int r = 0; r < NG; ++r) t += s_red[r][col];
                float o[1] = {t * sc};
                Elem<DT, 1>::store(a.Y, (int64_t)hv * a.ldy + gcol, o, 1, a.accumulate != 0, a.relu_h, (int64_t)hv * a.ldh + gcol);
            }
        }
        __syncthreads();
    }
}


// ---- edge-balanced kernel ------------------------------------------------------------------
// One workgroup owns up to kStreamMaxRows consecutive entries of the row list, but the work is split
// by EDGES, not by rows: the rows' neighbour lists are treated as one concatenated stream of E edges and
// each of the NG lane groups takes a contiguous E/NG stretch of it, LPR edges (one tile) per step.  A row
// that lies inside one stretch is summed and stored by that group; a row cut by a stretch boundary leaves
// its pieces in LDS ("carry" slots: at most a head piece and a tail piece per group), and after a barrier the
// pieces are added in stream order and stored.  So power-law rows cost no imbalance inside the workgroup,
// tiles are always full, and the result is a fixed-order sum (bit-reproducible).
// It serves the column-blocked route: the workgroup id carries (chunk, die) = (id / 8, id % 8); every row is cut to
// the die's column block through `seg`, and the unscaled float sums go to plane `die` of the partial buffer
// (a.Y, row index = position in the row list), not to the output matrix.
constexpr int kStreamMaxRows = 256;
#ifndef GNN_SPMM_STREAM_U
#define GNN_SPMM_STREAM_U 4        // row loads in flight per lane when a lane owns one 16-byte chunk of the row
#endif
#ifndef GNN_SPMM_STREAM_MINB
#define GNN_SPMM_STREAM_MINB 6     // workgroups per CU the register budget is cut for (L2-resident gathers
                                   // want resident wavefronts more than loads in flight: measured 4/6 > 8/4 > 16/3)
#endif
#ifndef GNN_SPMM_WG_EDGES
#define GNN_SPMM_WG_EDGES 8192     // edges one workgroup aims for when the host picks its row count
#endif

template <int DT, int VE, int LPR, int NCH, int U, bool SCALED>
__global__ __launch_bounds__(256, NCH == 1 ? GNN_SPMM_STREAM_MINB : 4) void spmm_stream_kernel(SpmmArgs a) {
    using E = Elem<DT, VE>;
    constexpr int RPW = kWave / LPR;
    constexpr int NG = 4 * RPW;
    constexpr int W = LPR * NCH * VE;  // feature columns per workgroup (grid.y blocks cover F)
    __shared__ int32_t s_start[kStreamMaxRows], s_voff[kStreamMaxRows + 1], s_v[kStreamMaxRows];
    __shared__ int32_t s_u_all[4][kWave], s_r_all[4][kWave];   // neighbour id and row slot of every staged edge
    __shared__ float s_w_all[4][kWave];                        // its scale factor (only with a neighbour scale)
    __shared__ float s_carry[NG * 2][W];
    __shared__ int32_t s_ctag[NG * 2];
    __shared__ int s_scan[4];
    const int tid = (int)threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int sub = lane / LPR, sl = lane % LPR;
    const int gi = wave * RPW + sub;
    int32_t* s_u = s_u_all[wave];
    int32_t* s_r = s_r_all[wave];
    float* s_w = s_w_all[wave];

    // ---- phase 0: row descriptors and the exclusive prefix of the row lengths
    const int rpw = a.rows_per_group;  // rows of the list per workgroup, <= kStreamMaxRows
    const int die = (int)(blockIdx.x % kDies);
    const int64_t chunk0 = (int64_t)(blockIdx.x / kDies) * rpw;
    const int n_chunk = (int)(((int64_t)a.n_active - chunk0) < rpw ? ((int64_t)a.n_active - chunk0) : rpw);
    float* const part = (float*)a.Y + (int64_t)die * a.n_active * a.ldy;
    int len = 0;
    if (tid < n_chunk) {
        const int32_t v = (int32_t)(chunk0 + tid);
        const int32_t* cut = a.seg + (int64_t)v * (a.n_blocks + 1) + a.block0 + die;
        const int32_t s = cut[0];
        const int32_t e = a.seg_end ? a.seg_end[(int64_t)v * a.n_blocks + a.block0 + die] : cut[1];
        s_v[tid] = v;
        s_start[tid] = s;
        len = e - s;
    }
    if (tid < NG * 2) s_ctag[tid] = -1;
    int n_edges;
    const int voff = block_exclusive_scan<256>(len, s_scan, &n_edges);
    if (tid < n_chunk) s_voff[tid] = voff;
    if (tid == 0) s_voff[n_chunk] = n_edges;
    __syncthreads();

    int per = (n_edges + NG - 1) / NG;
    per = (per + LPR - 1) / LPR * LPR;
    const int64_t lo64 = (int64_t)gi * per < n_edges ? (int64_t)gi * per : n_edges;
    const int lo = (int)lo64, hi = (int)(lo64 + per < n_edges ? lo64 + per : n_edges);  // this group's stretch of the stream

    int64_t col_off[NCH];
    bool col_ok[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        col_off[c] = (int64_t)blockIdx.y * W + (int64_t)(sl + c * LPR) * VE;
        col_ok[c] = col_off[c] < a.F;
    }
    // per-lane base address of its 16-byte chunk(s) of a row of X: column col_off, or column 0 for the lanes past
    // F (whose sums are never stored); a neighbour's row then adds its offset, staged in 16-byte units
    constexpr int ES = DT == GNN_F32 ? 4 : 2;
    const char* x_lane[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) x_lane[c] = (const char*)a.X + (col_ok[c] ? col_off[c] : 0) * ES;
    const uint32_t row16 = (uint32_t)(a.ldx * ES / 16);
    float acc[NCH][VE];
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int k = 0; k < VE; ++k) acc[c][k] = 0.f;

    // Row slot and position in col_idx of stream position t0 + sl (rows only move forward: r_hint).
    int r_hint = 0;
    auto locate = [&](int t0, int& r, int32_t& p) -> bool {
        const int t = t0 + sl;
        r = 0;
        p = 0;
        if (t >= hi) return false;
        int x = r_hint, y = n_chunk;  // s_voff[x] <= t < s_voff[y]
        while (y - x > 1) {
            const int m = (x + y) >> 1;
            if (s_voff[m] <= t) x = m;
            else y = m;
        }
        r_hint = x;
        r = x;
        p = s_start[x] + (t - s_voff[x]);
        return true;
    };

    int cur = -1;  // row slot the accumulators belong to (uniform over the group)
    auto flush = [&]() {
        const int b0 = s_voff[cur], b1 = s_voff[cur + 1];
        if (b0 >= lo && b1 <= hi) {  // the whole row lies in this stretch
            const int32_t v = s_v[cur];
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                if (col_ok[c]) {
                    const int64_t rest = (int64_t)a.F - col_off[c];
                    const int n_valid = rest >= VE ? VE : (int)rest;
                    store_part<VE>(part, (int64_t)v * a.ldy + col_off[c], acc[c], n_valid, a.accumulate != 0);
                }
            }
        } else {  // a piece: head (the row began in an earlier stretch) or tail (it goes on in the next one)
            const int slot = gi * 2 + (b0 < lo ? 0 : 1);
#pragma unroll
            for (int c = 0; c < NCH; ++c)
#pragma unroll
                for (int k = 0; k < VE; ++k) s_carry[slot][(sl + c * LPR) * VE + k] = acc[c][k];
            if (sl == 0) s_ctag[slot] = cur;
        }
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int k = 0; k < VE; ++k) acc[c][k] = 0.f;
    };

    // ---- phase 1: ids (and their scale factors, stored per edge by the prepare pass) are fetched two tiles ahead,
    // coalesced, each lane for its own edge, so the gather loop below touches global memory for feature rows only
    int t_c = lo;
    int r_c, r_n;
    int32_t p_c, p_n;
    // (a lane without an edge reads position 0 / vertex 0: the prefetches stay unconditional, see below)
    bool v_c = locate(t_c, r_c, p_c);
    bool v_n = locate(t_c + LPR, r_n, p_n);
    int32_t u_c = a.col_idx[p_c];
    int32_t u_n = a.col_idx[p_n];
    if (!v_c) u_c = 0;
    if (!v_n) u_n = 0;
    float w_c = 1.f, w_n = 1.f;
    if (SCALED) {
        w_c = a.edge_w[p_c];
        w_n = a.edge_w[p_n];
    }
    while (__ballot(t_c < hi) != 0ull) {  // uniform over the wave
        wave_lds_sync();  // the previous tile has been consumed
        // what is staged is the neighbour's row offset in 16-byte units (one multiply per lane and tile instead of
        // a 64-bit multiply per edge in the gather loop); 0 where the lane has no edge: a valid row all the same
        s_u[lane] = (int32_t)((uint32_t)u_c * row16);
        s_r[lane] = r_c;
        if (SCALED) s_w[lane] = w_c;
        int cnt = hi - t_c;
        cnt = cnt < 0 ? 0 : (cnt < LPR ? cnt : LPR);
        int cnt_max = cnt, cnt_min = cnt;
#pragma unroll
        for (int d = LPR; d < kWave; d <<= 1) {
            cnt_max = max(cnt_max, __shfl_xor(cnt_max, d, kWave));
            cnt_min = min(cnt_min, __shfl_xor(cnt_min, d, kWave));
        }
        // bit k of `starts`: edge k of this group's tile belongs to another row than the edge before it
        // (edge 0: than the accumulators); the gather loop reads one dword per edge (the id) and looks up
        // the row slot only where a row starts
        const int r_before = __shfl_up(r_c, 1, kWave);
        const bool start = v_c && r_c != (sl == 0 ? cur : r_before);
        const uint64_t starts = (__ballot(start) >> (sub * LPR)) & (LPR == 64 ? ~0ull : (1ull << (LPR & 63)) - 1ull);
        wave_lds_sync();
        // the prefetches go out right before this tile's gathers (everything older has been waited for by now)
        int r_nn;
        int32_t p_nn;
        const bool v_nn = locate(t_c + 2 * LPR, r_nn, p_nn);
        int32_t u_nn = a.col_idx[p_nn];
        float w_nn = 1.f;
        if (SCALED) w_nn = a.edge_w[p_nn];

#pragma unroll
        for (int k0 = 0; k0 < LPR; k0 += U) {
            if (k0 >= cnt_max) break;  // uniform over the wave
            // The loads are unconditional (a slot past the group's count holds row 0, a column past F reads
            // column 0: both valid addresses, the values are never used): with branches around them the compiler
            // waits for every load before issuing the next one.
            typename E::Raw x[U][NCH];
            float w[U];
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const uint64_t row_bytes = (uint64_t)(uint32_t)s_u[sub * LPR + k0 + j] << 4;
                w[j] = SCALED ? s_w[sub * LPR + k0 + j] : 1.f;
#pragma unroll
                for (int c = 0; c < NCH; ++c) x[j][c] = *(const typename E::Raw*)(x_lane[c] + row_bytes);
            }
            // common case, decided for the whole wave: every group has a full tile and no row starts inside this
            // round -> plain multiply-adds; else each edge checks its count and its row-start bit
            const bool round_has_start = ((starts >> k0) & ((1ull << U) - 1ull)) != 0ull;
            if (cnt_min == LPR && __ballot(round_has_start) == 0ull) {
#pragma unroll
                for (int j = 0; j < U; ++j)
#pragma unroll
                    for (int c = 0; c < NCH; ++c) E::fma(acc[c], w[j], x[j][c]);
            } else {
#pragma unroll
                for (int j = 0; j < U; ++j) {
                    if (k0 + j < cnt) {
                        if ((starts >> (k0 + j)) & 1ull) {
                            if (cur >= 0) flush();
                            cur = s_r[sub * LPR + k0 + j];
                        }
#pragma unroll
                        for (int c = 0; c < NCH; ++c) E::fma(acc[c], w[j], x[j][c]);
                    }
                }
            }
        }
        t_c += LPR;
        r_c = r_n; p_c = p_n; v_c = v_n; u_c = u_n; w_c = w_n;
        r_n = r_nn; p_n = p_nn; v_n = v_nn; u_n = v_nn ? u_nn : 0; w_n = w_nn;
    }
    if (cur >= 0) flush();
    __syncthreads();

    // ---- phase 2: rows cut by stretch boundaries - their pieces sit in consecutive carry slots
    for (int col = tid; col < W; col += 256) {
        const int64_t gcol = (int64_t)blockIdx.y * W + col;
        if (gcol >= a.F) continue;
        int tag = -1;
        float sum = 0.f;
        for (int q = 0; q <= NG * 2; ++q) {
            const int tq = q < NG * 2 ? s_ctag[q] : -2;
            if (tq == -1) continue;
            if (tq != tag) {
                if (tag >= 0) {
                    float o[1] = {sum};
                    const int64_t off = (int64_t)s_v[tag] * a.ldy + gcol;
                    store_part<1>(part, off, o, 1, a.accumulate != 0);
                }
                tag = tq;
                sum = 0.f;
            }
            if (tq >= 0) sum += s_carry[q][col];
        }
    }
    // ---- phase 3: rows without any edge are zero (they never show up in the stream)
    if (!a.accumulate) {
        for (int r = gi; r < n_chunk; r += NG) {
            if (s_voff[r + 1] != s_voff[r]) continue;
            const int32_t v = s_v[r];
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                if (col_ok[c]) {
                    float o[VE];
#pragma unroll
                    for (int k = 0; k < VE; ++k) o[k] = 0.f;
                    const int64_t rest = (int64_t)a.F - col_off[c];
                    const int n_valid = rest >= VE ? VE : (int)rest;
                    store_part<VE>(part, (int64_t)v * a.ldy + col_off[c], o, n_valid, false);
                }
            }
        }
    }
}

template <int DT, int VE, int LPR, int NCH>
static int32_t launch_stream(const SpmmArgs& a, int64_t avg_row, hipStream_t stream) {
    constexpr int U = NCH == 1 ? GNN_SPMM_STREAM_U : (NCH == 2 ? 4 : (NCH == 3 ? 3 : 2));
    constexpr int W = LPR * NCH * VE;
    // rows per workgroup: about GNN_SPMM_WG_EDGES edges, while the launch keeps a few thousand workgroups
    SpmmArgs b = a;
    int64_t rows = (int64_t)GNN_SPMM_WG_EDGES / (avg_row < 1 ? 1 : avg_row);
    const int64_t cap = (int64_t)a.n_active * kDies / 4096;
    if (rows > cap) rows = cap;
    b.rows_per_group = (int32_t)(rows < 16 ? 16 : (rows > kStreamMaxRows ? kStreamMaxRows : rows));
    const int64_t n_chunks = ((int64_t)a.n_active + b.rows_per_group - 1) / b.rows_per_group;
    dim3 grid((unsigned)(n_chunks * kDies), (unsigned)((a.F + W - 1) / W));
    if (a.edge_w) spmm_stream_kernel<DT, VE, LPR, NCH, U, true><<<grid, 256, 0, stream>>>(b);
    else spmm_stream_kernel<DT, VE, LPR, NCH, U, false><<<grid, 256, 0, stream>>>(b);
    GNN_LAUNCH_CHECK("spmm_stream_kernel");
    return GNN_OK;
}

template <int DT, int VE, int LPR, int NCH, bool FILTER>
static int32_t launch_rows(const SpmmArgs& a, hipStream_t stream) {
    constexpr int U = NCH == 1 ? (LPR < 16 ? 4 : (LPR < 64 ? GNN_SPMM_U_NARROW : GNN_SPMM_U_WIDE)) : (NCH == 2 ? 4 : (NCH == 3 ? 3 : 2));
    constexpr int NG = 4 * (kWave / LPR);
    constexpr int W = LPR * NCH * VE;
    // chunk size: as large as possible (better balance inside a workgroup) while the launch still
    // has about 16 workgroups per CU
    SpmmArgs b = a;
    int rpg = (int)((int64_t)a.n_active / ((int64_t)NG * 4096));
    constexpr int kMaxRpg = kRowsPerGroup * NG <= kMaxChunk ? kRowsPerGroup : kMaxChunk / NG;
    b.rows_per_group = rpg < 1 ? 1 : (rpg > kMaxRpg ? kMaxRpg : rpg);
    const int rpb = NG * b.rows_per_group;
    dim3 grid((unsigned)(((int64_t)a.n_active + rpb - 1) / rpb), (unsigned)((a.F + W - 1) / W));
    spmm_rows_kernel<DT, VE, LPR, NCH, U, FILTER><<<grid, 256, 0, stream>>>(b);
    GNN_LAUNCH_CHECK("spmm_rows_kernel");
    return GNN_OK;
}

// Column-block boundaries of a FILTERED call: bounds[j], j = 0 .. n_blocks, split the neighbour-id range so that
// every block holds the same number of ACTIVE vertices (0 <= dist <= max_dist) - only those are ever gathered, and
// they need not be spread evenly over the id range (after a (distance, id) renumbering they are a prefix).
// One workgroup of 1024 threads: per-thread counts over contiguous id chunks, a block scan, then the thread whose
// chunk contains the j-th quantile walks it to the exact id.
__global__ __launch_bounds__(1024) void spmm_bounds_kernel(const int32_t* __restrict__ dist, int32_t max_dist, int32_t n_cols,
                                                            int32_t n_blocks, int32_t* __restrict__ bounds) {
    __shared__ int s_part[16];
    const int64_t chunk = ((int64_t)n_cols + 1023) / 1024;
    const int64_t lo = (int64_t)threadIdx.x * chunk, hi = lo + chunk < n_cols ? lo + chunk : n_cols;
    int cnt = 0;
    for (int64_t u = lo; u < hi; ++u) {
        const int32_t d = dist[u];
        cnt += d >= 0 && d <= max_dist;
    }
    int total;
    const int before = block_exclusive_scan<1024>(cnt, s_part, &total);
    if (threadIdx.x == 0) {
        bounds[0] = 0;
        bounds[n_blocks] = n_cols;
    }
    // boundary j sits before the active vertex of rank ceil(j * total / n_blocks) (ranks from 0)
    for (int j = 1; j < n_blocks; ++j) {
        const int64_t want = ((int64_t)j * total + n_blocks - 1) / n_blocks;
        if (total == 0) {
            if (threadIdx.x == 0) bounds[j] = (int32_t)((int64_t)j * n_cols / n_blocks);
        } else if (want >= before && want < (int64_t)before + cnt) {
            int64_t rank = before;
            for (int64_t u = lo; u < hi; ++u) {
                const int32_t d = dist[u];
                if (d >= 0 && d <= max_dist) {
                    if (rank == want) {
                        bounds[j] = (int32_t)u;
                        break;
                    }
                    ++rank;
                }
            }
        } else if (want >= total && threadIdx.x == 0) {
            bounds[j] = n_cols;
        }
    }
}

// Cut points of every listed row at the column-block boundaries (rows sorted by column): seg[r][j] = first position
// of row r whose column is >= the j-th boundary (bounds[j] if given, else j * block_size); seg[r][0] = start,
// seg[r][n_blocks] = end - or, with limit < n_cols, the first position whose column is >= limit (the entries past it
// are never gathered), and no boundary lies above limit.
__global__ __launch_bounds__(256) void spmm_seg_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                                                        const int32_t* __restrict__ rows, int32_t n_active, int32_t n_blocks,
                                                        int32_t block_size, const int32_t* __restrict__ bounds, int32_t limit,
                                                        int32_t n_cols, int32_t* __restrict__ seg) {
    const int64_t total = (int64_t)n_active * (n_blocks + 1);
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int32_t r = (int32_t)(i / (n_blocks + 1)), j = (int32_t)(i % (n_blocks + 1));
        const int32_t v = rows ? rows[r] : r;
        int32_t lo = row_ptr[v], hi = row_ptr[v + 1];
        if (j == n_blocks) {
            lo = limit < n_cols ? row_lower_bound(col_idx, lo, hi, limit) : hi;
        } else if (j > 0) {
            int64_t bound = bounds ? (int64_t)bounds[j] : (int64_t)j * block_size;
            bound = bound < limit ? bound : limit;
            lo = row_lower_bound(col_idx, lo, hi, bound);
        }
        seg[i] = lo;
    }
}

// Per-edge preparation of the column-blocked route, done once per call instead of once per feature slab: every
// (row, block) segment is copied to `ids` at its own position - with a dist filter (backward) the neighbours that
// fail the test are squeezed out, seg_end[r][j] = where the kept ones end - and with a neighbour scale the factor of
// every kept neighbour goes to `w` at the same position (the random 4-byte gathers of the scale vector happen here,
// once; the stream kernel then reads ids and factors coalesced).  One group of 16 lanes per segment.
__global__ __launch_bounds__(256) void spmm_prepare_kernel(const int32_t* __restrict__ col_idx, const int32_t* __restrict__ seg,
                                                            const int32_t* __restrict__ dist, int32_t max_dist,
                                                            const float* __restrict__ nbr_scale, int64_t n_segments, int32_t n_blocks,
                                                            int32_t* __restrict__ ids, float* __restrict__ w, int32_t* __restrict__ seg_end) {
    constexpr int LPG = 16;
    const int lane = lane_id(), sub = lane / LPG, sl = lane % LPG;
    const int64_t groups = (int64_t)gridDim.x * (blockDim.x / LPG);
    for (int64_t sgm = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / LPG; sgm < n_segments; sgm += groups) {
        const int64_t r = sgm / n_blocks;
        const int32_t j = (int32_t)(sgm % n_blocks);
        const int32_t lo = seg[r * (n_blocks + 1) + j], hi = seg[r * (n_blocks + 1) + j + 1];
        int32_t out = lo;
        // kT tiles of 16 entries per step: all their id loads go out together, then all dist / scale loads, so a
        // typical segment (a few tiles) pays each memory latency once instead of once per tile
        constexpr int kT = 4;
        for (int32_t p = lo; p < hi; p += kT * LPG) {
            int32_t u[kT], d[kT];
            float f[kT];
            bool valid[kT];
#pragma unroll
            for (int t = 0; t < kT; ++t) {
                valid[t] = p + t * LPG + sl < hi;
                u[t] = valid[t] ? col_idx[p + t * LPG + sl] : 0;
            }
#pragma unroll
            for (int t = 0; t < kT; ++t) {
                d[t] = dist ? dist[u[t]] : 0;          // u = 0 where the lane has no entry: a valid index
                f[t] = nbr_scale ? nbr_scale[u[t]] : 1.f;
            }
#pragma unroll
            for (int t = 0; t < kT; ++t) {
                const bool keep = valid[t] && d[t] >= 0 && d[t] <= (dist ? max_dist : 0);
                const uint64_t kept = (__ballot(keep) >> (sub * LPG)) & 0xffffull;
                if (keep) {
                    const int32_t q = out + __popcll(kept & ((1ull << sl) - 1ull));
                    ids[q] = u[t];
                    if (nbr_scale) w[q] = f[t];
                }
                out += __popcll(kept);
            }
        }
        if (sl == 0) seg_end[sgm] = out;
    }
}

// Y[v, c] (+)= out_scale[v] * (plane 0 + plane 1 + ... + plane 7)[r, c], v = rows[r]: planes added in die order.
// One thread per four columns; part rows are 16-byte aligned, and so are the rows of Y (vector route only).
template <int DT>
__global__ __launch_bounds__(256) void spmm_sum_parts_kernel(const float* __restrict__ part, int64_t ldp, const int32_t* __restrict__ rows,
                                                              int32_t n_active, int32_t F, void* __restrict__ Y, int64_t ldy,
                                                              const float* __restrict__ out_scale, int32_t accumulate, const void* __restrict__ relu_h, int64_t ldh) {
    const int32_t f4 = (F + 3) / 4;
    const int64_t total = (int64_t)n_active * f4;
    const int64_t plane = (int64_t)n_active * ldp;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int32_t r = (int32_t)(i / f4), c = (int32_t)(i % f4) * 4;
        const int32_t v = rows ? rows[r] : r;
        float4 t = *(const float4*)(part + (int64_t)r * ldp + c);
#pragma unroll
        for (int d = 1; d < kDies; ++d) {
            const float4 q = *(const float4*)(part + d * plane + (int64_t)r * ldp + c);
            t.x += q.x; t.y += q.y; t.z += q.z; t.w += q.w;
        }
        const float sc = out_scale ? out_scale[v] : 1.f;
        float o[4] = {t.x * sc, t.y * sc, t.z * sc, t.w * sc};
        const int n_valid = F - c >= 4 ? 4 : F - c;
        const int64_t off = (int64_t)v * ldy + c;
        // the stored value is zeroed where relu_h (same rows and columns as Y) is <= 0; relu_h == Y: where it is <= 0 itself
        const bool self = relu_h == (const void*)Y;
        bool pass[4] = {true, true, true, true};
        if (relu_h && !self) {
            for (int k = 0; k < n_valid; ++k) pass[k] = Elem<DT, 1>::to_float(Elem<DT, 1>::load(relu_h, (int64_t)v * ldh + c + k)) > 0.f;
        }
        if (accumulate) {
            if (DT == GNN_F32) {
                const float* y = (const float*)Y + off;
                for (int k = 0; k < n_valid; ++k) o[k] += y[k];
            } else {
                const uint16_t* y = (const uint16_t*)Y + off;
                for (int k = 0; k < n_valid; ++k) o[k] += bf16_to_f32(y[k]);
            }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = (self ? o[k] > 0.f : pass[k]) ? o[k] : 0.f;
        if (DT == GNN_F32) {
            float* y = (float*)Y + off;
            if (n_valid == 4) *(float4*)y = make_float4(o[0], o[1], o[2], o[3]);
            else
                for (int k = 0; k < n_valid; ++k) y[k] = o[k];
        } else {
            uint16_t* y = (uint16_t*)Y + off;
            if (n_valid == 4) *(uint2*)y = make_uint2(pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3]));
            else
                for (int k = 0; k < n_valid; ++k) y[k] = f32_to_bf16(o[k]);
        }
    }
}

// Y[v, 0:F] = bias[0:F] for the listed rows: the starting value of an aggregation that has no self term under it.
template <int DT>
__global__ __launch_bounds__(256) void spmm_bias_rows_kernel(const int32_t* __restrict__ rows, int32_t n_active, const float* __restrict__ bias,
                                                              void* __restrict__ Y, int64_t ldy, int32_t F) {
    const int64_t total = (int64_t)n_active * F;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int32_t i = (int32_t)(t / F), c = (int32_t)(t % F);
        const int64_t v = rows ? (int64_t)rows[i] : i;
        if (DT == GNN_F32) ((float*)Y)[v * ldy + c] = bias[c];
        else ((uint16_t*)Y)[v * ldy + c] = f32_to_bf16(bias[c]);
    }
}

// Xs[u, 0:F] = scale[u] * X[u, 0:F] for every row of the gathered matrix (16-byte aligned rows): with a neighbour scale
// the column-blocked route gathers from this copy, so its inner loop needs no per-edge factor.
template <int DT>
__global__ __launch_bounds__(256) void spmm_scale_rows_kernel(const void* __restrict__ X, int64_t ldx, int32_t n_rows, int32_t F,
                                                              const float* __restrict__ scale, void* __restrict__ Xs) {
    using E = Elem<DT, DT == GNN_F32 ? 4 : 8>;
    constexpr int VE = E::VE;
    const int vpr = (F + VE - 1) / VE;
    const int64_t total = (int64_t)n_rows * vpr;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t u = t / vpr;
        const int64_t off = u * ldx + (t % vpr) * VE;
        float acc[VE];
#pragma unroll
        for (int e = 0; e < VE; ++e) acc[e] = 0.f;
        E::fma(acc, scale[u], E::load(X, off));
        E::store(Xs, off, acc, VE, false);
    }
}

// ---- does workgroup i run on compute die i mod 8? --------------------------------------------------------------
// The column-blocked route rests on it (correctness does not: with another dispatch order the sums are the same, only
// the reason for the route is gone).  Checked once per device, at the first call that would take the route: a 16 x 4
// grid of one-wave workgroups records the die (XCC) id each of them ran on; the route is taken only if the first eight
// ids are eight different dies and workgroup i (in dispatch order: x fastest) repeats the die of workgroup i mod 8.
constexpr int kProbeX = 16, kProbeY = 4;
static __device__ int32_t g_die_probe[kProbeX * kProbeY];

__global__ __launch_bounds__(64) void die_probe_kernel(int32_t* __restrict__ out) {
    uint32_t x;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(x));   // bits 3:0: the die this wavefront runs on
    if (threadIdx.x == 0) out[blockIdx.y * gridDim.x + blockIdx.x] = (int32_t)(x & 0xfu);
}

static int32_t probe_die_ids(int32_t* ids_host) {
    void* p = nullptr;
    GNN_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(g_die_probe)));
    die_probe_kernel<<<dim3(kProbeX, kProbeY), 64, 0, (hipStream_t)0>>>((int32_t*)p);
    GNN_LAUNCH_CHECK("die_probe_kernel");
    GNN_HIP(hipMemcpy(ids_host, p, sizeof(int32_t) * kProbeX * kProbeY, hipMemcpyDeviceToHost));   // waits for the kernel
    return GNN_OK;
}

static bool die_ids_round_robin(const int32_t* ids) {
    uint32_t seen = 0;
    for (int i = 0; i < kDies; ++i) {
        if (ids[i] < 0 || ids[i] >= kDies) return false;
        seen |= 1u << ids[i];
    }
    if (seen != (1u << kDies) - 1u) return false;
    for (int i = kDies; i < kProbeX * kProbeY; ++i)
        if (ids[i] != ids[i % kDies]) return false;
    return true;
}

// 1: the mapping holds on the current device, 0: it does not (or could not be probed); probed at the first question
static int die_mapping_holds() {
    static std::mutex mu;
    static int state[64];   // per device: 0 unknown, 1 holds, 2 does not
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    std::lock_guard<std::mutex> lock(mu);
    if (state[dev] == 0) {
        int32_t ids[kProbeX * kProbeY];
        state[dev] = (probe_die_ids(ids) == GNN_OK && die_ids_round_robin(ids)) ? 1 : 2;
    }
    return state[dev] == 1;
}

// The column-blocked route's shape for one call; passes == 0: the route does not apply.
struct BlockedPlan {
    int passes = 0;
    int n_blocks = 0;
    int32_t block_size = 0;
    int64_t ldp = 0;          // leading dimension of a partial plane, in floats
    size_t seg_bytes = 0, part_bytes = 0;
    size_t end_bytes = 0, ids_bytes = 0;   // with a filter or a neighbour scale: segment ends and the (compacted) copy of the ids
    size_t xs_bytes = 0;                   // fp32 with a neighbour scale: the gathered matrix with its rows scaled
    size_t w_bytes = 0;                    // bf16 with a neighbour scale: the factor of every copied id
    int64_t avg_seg = 0;      // average neighbours of a row inside one column block
    int32_t n_cols = 0;
    int32_t limit = 0;        // neighbour ids >= limit are never gathered (n_cols without a source prefix)
    size_t bounds_bytes = 0;  // with a filter: the column-block boundaries (balanced over the active vertices)
};

static BlockedPlan plan_blocked(const gnn_csr* g, int32_t n_active, int32_t F, int64_t row_bytes, bool vec_ok, bool filter,
                                bool scaled, bool f32, int32_t src_prefix) {
    BlockedPlan p;
    // with a source prefix only the rows [0, src_prefix) of the gathered matrix are ever read
    const int32_t n_src = (src_prefix >= 0 && src_prefix < g->n_cols) ? src_prefix : g->n_cols;
    // the stream kernel addresses the gathered matrix with 32-bit offsets in 16-byte units: 64 GB at most
    if ((int64_t)g->n_cols * row_bytes >= ((int64_t)1 << 36)) return p;
    if (!vec_ok || !(g->flags & GNN_CSR_SORTED_COLUMNS) || g->n_rows <= 0 || n_active < 4096) return p;
    if (g->edge_keep != nullptr) return p;  // the per-layer edge mask is only known to the one-launch route
    const int64_t slab = (int64_t)n_src * kSlabBytes;
    if (slab < (int64_t)GNN_SPMM_BLOCKED_MIN_SLAB) return p;
    const int passes = (int)((slab + kDies * (int64_t)GNN_SPMM_DIE_BYTES - 1) / (kDies * (int64_t)GNN_SPMM_DIE_BYTES));
    const int n_blocks = kDies * passes;
    // average kept length of a row: its entries spread over the id range like the vertices do
    const int64_t avg_row = (int64_t)((double)g->nnz / g->n_rows * ((double)n_src / g->n_cols));
    if (avg_row < (int64_t)GNN_SPMM_BLOCKED_MIN_SEG * n_blocks) return p;
    if (!die_mapping_holds()) return p;     // workgroup i is not on die i mod 8 here: the route has lost its reason
    p.passes = passes;
    p.n_blocks = n_blocks;
    p.avg_seg = avg_row / n_blocks;
    p.block_size = (int32_t)(((int64_t)n_src + n_blocks - 1) / n_blocks);
    p.limit = n_src;
    p.ldp = ((int64_t)F + 7) / 8 * 8;
    p.seg_bytes = (size_t)n_active * (n_blocks + 1) * sizeof(int32_t);
    p.part_bytes = (size_t)kDies * n_active * p.ldp * sizeof(float);
    // A neighbour scale: fp32 gathers from a copy of the matrix with scaled rows (one rounding more per element,
    // far inside the fp32 tolerance); bf16 would lose too much in a rounded copy and keeps a factor per edge.
    if (filter || (scaled && !f32)) {
        p.end_bytes = (size_t)n_active * n_blocks * sizeof(int32_t);
        p.ids_bytes = (size_t)g->nnz * sizeof(int32_t);
    }
    if (scaled && f32) p.xs_bytes = (size_t)n_src * (size_t)row_bytes;
    if (scaled && !f32) p.w_bytes = (size_t)g->nnz * sizeof(float);
    if (filter) p.bounds_bytes = ((size_t)n_blocks + 1) * sizeof(int32_t);
    p.n_cols = g->n_cols;
    return p;
}

template <int DT, bool FILTER>
static int32_t run_blocked(const SpmmArgs& a, const BlockedPlan& p, void* ws, hipStream_t stream) {
    constexpr int VE = DT == GNN_F32 ? 4 : 8;
    WsCarver carve(ws);
    int32_t* seg = carve.take<int32_t>(p.seg_bytes / sizeof(int32_t));
    float* part = carve.take<float>(p.part_bytes / sizeof(float));
    const bool prescale = a.nbr_scale != nullptr && DT == GNN_F32, per_edge = a.nbr_scale != nullptr && DT != GNN_F32;
    const bool prepare = FILTER || per_edge;
    int32_t* seg_end = prepare ? carve.take<int32_t>(p.end_bytes / sizeof(int32_t)) : nullptr;
    int32_t* ids = prepare ? carve.take<int32_t>(p.ids_bytes / sizeof(int32_t)) : nullptr;
    char* xs = prescale ? carve.take<char>(p.xs_bytes) : nullptr;
    float* edge_w = per_edge ? carve.take<float>(p.w_bytes / sizeof(float)) : nullptr;
    int32_t* bounds = FILTER ? carve.take<int32_t>((size_t)p.n_blocks + 1) : nullptr;
    if (FILTER) {
        spmm_bounds_kernel<<<1, 1024, 0, stream>>>(a.dist, a.max_dist, p.n_cols, p.n_blocks, bounds);
        GNN_LAUNCH_CHECK("spmm_bounds_kernel");
    }
    spmm_seg_kernel<<<grid_for((int64_t)a.n_active * (p.n_blocks + 1), 256, 1 << 16), 256, 0, stream>>>(
        a.row_ptr, a.col_idx, a.rows, a.n_active, p.n_blocks, p.block_size, bounds, p.limit, p.n_cols, seg);
    GNN_LAUNCH_CHECK("spmm_seg_kernel");
    SpmmArgs b = a;
    if (prescale) {
        // the neighbour scale is applied once per row of the gathered matrix, not once per edge and slab
        spmm_scale_rows_kernel<DT><<<grid_for((int64_t)p.limit * ((a.F + VE - 1) / VE), 256, 1 << 16), 256, 0, stream>>>(
            a.X, a.ldx, p.limit, a.F, a.nbr_scale, xs);
        GNN_LAUNCH_CHECK("spmm_scale_rows_kernel");
        b.X = xs;
        b.nbr_scale = nullptr;
    }
    if (prepare) {
        const int64_t n_segments = (int64_t)a.n_active * p.n_blocks;
        spmm_prepare_kernel<<<grid_for(n_segments * 16, 256, 1 << 18), 256, 0, stream>>>(
            a.col_idx, seg, FILTER ? a.dist : nullptr, a.max_dist, per_edge ? a.nbr_scale : nullptr, n_segments, p.n_blocks, ids, edge_w,
            seg_end);
        GNN_LAUNCH_CHECK("spmm_prepare_kernel");
        b.col_idx = ids;
        b.seg_end = seg_end;
        b.edge_w = edge_w;
        b.dist = nullptr;
    }
    b.seg = seg;
    b.n_blocks = p.n_blocks;
    b.Y = part;
    b.ldy = p.ldp;
    b.out_scale = nullptr;
    for (int pass = 0; pass < p.passes; ++pass) {
        b.block0 = pass * kDies;
        b.accumulate = pass > 0;
        GNN_CHECK((launch_stream<DT, VE, 16, 1>(b, p.avg_seg, stream)));
    }
    spmm_sum_parts_kernel<DT><<<grid_for((int64_t)a.n_active * ((a.F + 3) / 4), 256, 1 << 16), 256, 0, stream>>>(
        part, p.ldp, a.rows, a.n_active, a.F, a.Y, a.ldy, a.out_scale, a.accumulate, a.relu_h, a.ldh);
    GNN_LAUNCH_CHECK("spmm_sum_parts_kernel");
    return GNN_OK;
}

template <int DT, bool FILTER>
static int32_t dispatch(const SpmmArgs& a, bool vec_ok, hipStream_t stream) {
    constexpr int VE = DT == GNN_F32 ? 4 : 8;
    const int F = a.F;
    // any alignment / leading dimension: element-wise lanes, 256 columns per workgroup
    if (!vec_ok) return launch_rows<DT, 1, 64, 4, FILTER>(a, stream);
    // Narrow outputs (class scores, a layer in the exchanged order).  A tile of the row kernel is as long as the lanes
    // that span a row, and a short tile pays the per-tile work (staging, ballots, row claims) for few neighbours: rows
    // narrower than 16 vectors of 16 bytes keep their 16 lanes and 16-neighbour tiles and take fewer bytes per lane
    // instead (measured on 64-byte rows: 8 lanes x 16 bytes 2.45 ms, 16 lanes x 4 bytes 1.81 ms).
    if (DT == GNN_BF16) {
        if (F <= 16) return launch_rows<GNN_BF16, 1, 16, 1, FILTER>(a, stream);
        if (F <= 32) return launch_rows<GNN_BF16, 2, 16, 1, FILTER>(a, stream);
        if (F <= 64) return launch_rows<GNN_BF16, 4, 16, 1, FILTER>(a, stream);
    } else {
        if (F <= 16) return launch_rows<GNN_F32, 1, 16, 1, FILTER>(a, stream);
        if (F <= 32) return launch_rows<GNN_F32, 2, 16, 1, FILTER>(a, stream);
    }
    if (F <= 16 * VE) return launch_rows<DT, VE, 16, 1, FILTER>(a, stream);
    if (F <= 32 * VE) return launch_rows<DT, VE, 32, 1, FILTER>(a, stream);
    if (F <= 64 * VE) return launch_rows<DT, VE, 64, 1, FILTER>(a, stream);
    if (F <= 128 * VE) return launch_rows<DT, VE, 64, 2, FILTER>(a, stream);
    return launch_rows<DT, VE, 64, 3, FILTER>(a, stream);
}

static int32_t spmm_common(const gnn_csr* g, const char* gname, const int32_t* rows, int32_t n_active, const int32_t* dist,
                           int32_t max_dist, int32_t src_prefix, const void* X, int64_t ldx, void* Y, int64_t ldy, int32_t F, int32_t dtype,
                           const float* out_scale, const float* nbr_scale, int32_t accumulate, const void* relu_h, int64_t ldh,
                           void* ws, size_t* ws_bytes, hipStream_t stream, const float* start_bias = nullptr) {
    GNN_CHECK(check_csr(g, gname));
    GNN_REQUIRE(n_active >= 0, GNN_ERR_INVALID_ARG, "negative row count");
    GNN_REQUIRE(rows != nullptr || n_active <= g->n_rows, GNN_ERR_SHAPE, "n_active %d exceeds n_rows %d", n_active, g->n_rows);
    GNN_REQUIRE(dtype == GNN_F32 || dtype == GNN_BF16, GNN_ERR_UNSUPPORTED, "unknown dtype %d", dtype);
    GNN_REQUIRE(F >= 0, GNN_ERR_INVALID_ARG, "F < 0");
    GNN_REQUIRE(ldx >= F && ldy >= F, GNN_ERR_SHAPE, "leading dimension smaller than F = %d", F);
    const int ve = dtype == GNN_F32 ? 4 : 8;
    GNN_REQUIRE(relu_h == nullptr || ldh >= F, GNN_ERR_SHAPE, "ld_relu smaller than F = %d", F);
    const bool vec_ok = ((uintptr_t)X % 16 == 0) && ((uintptr_t)Y % 16 == 0) && ldx % ve == 0 && ldy % ve == 0 &&
                        (relu_h == nullptr || ((uintptr_t)relu_h % 16 == 0 && ldh % ve == 0));
    GNN_REQUIRE(src_prefix >= -1, GNN_ERR_INVALID_ARG, "src_prefix %d: -1 or a vertex count", src_prefix);
    // A source prefix that leaves something out: rows sorted by column are cut at that id (no test per entry), rows in
    // any order get the test in the filter.
    const bool use_prefix = src_prefix >= 0 && src_prefix < g->n_cols;
    const bool sorted = (g->flags & GNN_CSR_SORTED_COLUMNS) != 0;
    const int32_t cut_id = (use_prefix && sorted) ? src_prefix : -1, id_limit = (use_prefix && !sorted) ? src_prefix : -1;
    const bool filter = dist != nullptr || g->edge_keep != nullptr || id_limit >= 0;
    BlockedPlan plan;
    if (ws_bytes != nullptr) {
        if (n_active > 0 && F > 0) plan = plan_blocked(g, n_active, F, ldx * (dtype == GNN_F32 ? 4 : 2), vec_ok, filter, nbr_scale != nullptr,
                                                            dtype == GNN_F32, cut_id);
        WsCarver measure(nullptr);
        if (plan.passes > 0) {
            measure.take<char>(plan.seg_bytes);
            measure.take<char>(plan.part_bytes);
            if (plan.end_bytes) {
                measure.take<char>(plan.end_bytes);
                measure.take<char>(plan.ids_bytes);
            }
            if (plan.xs_bytes) measure.take<char>(plan.xs_bytes);
            if (plan.w_bytes) measure.take<char>(plan.w_bytes);
            if (plan.bounds_bytes) measure.take<char>(plan.bounds_bytes);
        }
        bool query_only = false;
        GNN_CHECK(ws_protocol(ws, ws_bytes, measure.used, &query_only));
        if (query_only) return GNN_OK;
    }
    if (n_active == 0 || F == 0) return GNN_OK;
    GNN_REQUIRE(X != nullptr && Y != nullptr, GNN_ERR_INVALID_ARG, "X or Y is NULL");
    if (start_bias != nullptr) {
        // no self term under the sum (GCN in the exchanged order): the listed rows start from the bias
        const int grid = grid_for((int64_t)n_active * F, 256, 1 << 14);
        if (dtype == GNN_F32) spmm_bias_rows_kernel<GNN_F32><<<grid, 256, 0, stream>>>(rows, n_active, start_bias, Y, ldy, F);
        else spmm_bias_rows_kernel<GNN_BF16><<<grid, 256, 0, stream>>>(rows, n_active, start_bias, Y, ldy, F);
        GNN_LAUNCH_CHECK("spmm_bias_rows_kernel");
    }

    SpmmArgs a;
    a.row_ptr = g->row_ptr; a.col_idx = g->col_idx; a.rows = rows; a.n_active = n_active;
    a.X = X; a.ldx = ldx; a.Y = Y; a.ldy = ldy; a.F = F;
    a.out_scale = out_scale; a.nbr_scale = nbr_scale; a.dist = dist; a.max_dist = dist ? max_dist : INT32_MAX;
    a.edge_keep = g->edge_keep;
    a.cut_id = cut_id; a.id_limit = id_limit;
    a.accumulate = accumulate;
    a.relu_h = relu_h; a.ldh = ldh;
    a.rows_per_group = 1;
    {
        const int64_t row_bytes = ldx * (dtype == GNN_F32 ? 4 : 2);
        const bool small = g->n_cols < (1 << 24) && row_bytes < (1 << 24) && (int64_t)g->n_cols * row_bytes < ((int64_t)1 << 32);
        a.x_row_bytes = small ? (uint32_t)row_bytes : 0u;
    }
    a.seg = nullptr; a.seg_end = nullptr; a.edge_w = nullptr; a.n_blocks = 0; a.block0 = 0;

    if (plan.passes > 0) {
        if (dtype == GNN_F32) return filter ? run_blocked<GNN_F32, true>(a, plan, ws, stream) : run_blocked<GNN_F32, false>(a, plan, ws, stream);
        return filter ? run_blocked<GNN_BF16, true>(a, plan, ws, stream) : run_blocked<GNN_BF16, false>(a, plan, ws, stream);
    }
    if (dtype == GNN_F32) return filter ? dispatch<GNN_F32, true>(a, vec_ok, stream) : dispatch<GNN_F32, false>(a, vec_ok, stream);
    return filter ? dispatch<GNN_BF16, true>(a, vec_ok, stream) : dispatch<GNN_BF16, false>(a, vec_ok, stream);
}

}  // namespace gnnhot

using namespace gnnhot;

extern "C" int32_t gnn_die_mapping(int32_t* xcc_ids_host, int32_t n_ids, int32_t* holds_host) {
    GNN_REQUIRE(n_ids >= 0 && (xcc_ids_host != nullptr || n_ids == 0), GNN_ERR_INVALID_ARG, "xcc_ids_host is NULL");
    int32_t ids[kProbeX * kProbeY];
    GNN_CHECK(probe_die_ids(ids));
    for (int i = 0; i < n_ids && i < kProbeX * kProbeY; ++i) xcc_ids_host[i] = ids[i];
    if (holds_host != nullptr) *holds_host = die_ids_round_robin(ids) ? 1 : 0;
    return GNN_OK;
}

extern "C" int32_t gnn_masked_spmm_fwd(const gnn_csr* g, const int32_t* rows, int32_t n_active, const void* X, int64_t ldx,
                                       void* Y, int64_t ldy, int32_t F, int32_t dtype, const float* row_scale,
                                       const float* col_scale, void* ws, size_t* ws_bytes, void* stream) {
    return spmm_common(g, "g", rows, n_active, nullptr, 0, -1, X, ldx, Y, ldy, F, dtype, row_scale, col_scale, 0, nullptr, 0, ws,
                       ws_bytes, (hipStream_t)stream);
}

extern "C" int32_t gnn_masked_spmm_fwd_add(const gnn_csr* g, const int32_t* rows, int32_t n_active, const void* X, int64_t ldx,
                                           void* Y, int64_t ldy, int32_t F, int32_t dtype, const float* row_scale,
                                           const float* col_scale, const float* bias, int32_t relu, void* ws, size_t* ws_bytes,
                                           void* stream) {
    GNN_REQUIRE(relu == 0 || relu == 1, GNN_ERR_INVALID_ARG, "relu must be 0 or 1");
    // the output matrix as its own mask stands for a ReLU of what is stored
    return spmm_common(g, "g", rows, n_active, nullptr, 0, -1, X, ldx, Y, ldy, F, dtype, row_scale, col_scale, 1, relu ? Y : nullptr, ldy, ws,
                       ws_bytes, (hipStream_t)stream, bias);
}

extern "C" int32_t gnn_masked_spmm_bwd(const gnn_csr* gT, const int32_t* out_rows, int32_t n_out, const int32_t* dist,
                                       int32_t max_active_dist, int32_t src_prefix, const void* dY, int64_t lddy, void* dX, int64_t lddx, int32_t F,
                                       int32_t dtype, const float* row_scale, const float* col_scale, int32_t accumulate,
                                       const void* relu_H, int64_t ld_relu, void* ws, size_t* ws_bytes, void* stream) {
    GNN_REQUIRE(accumulate == 0 || accumulate == 1, GNN_ERR_INVALID_ARG, "accumulate must be 0 or 1");
    return spmm_common(gT, "gT", out_rows, n_out, dist, max_active_dist, src_prefix, dY, lddy, dX, lddx, F, dtype, col_scale, row_scale,
                       accumulate, relu_H, ld_relu, ws, ws_bytes, (hipStream_t)stream);
}
