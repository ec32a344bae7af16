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
// 16-byte loads in flight per lane.  Groups claim rows dynamically inside a workgroup's chunk.  Rows longer than kHubDegree
// (power-law hubs) are split over all wavefronts of the workgroup and the partial sums are
// reduced through LDS in a fixed order, inside the same launch.
#include "common.h"

namespace gnnhot {

// independent row loads in flight per lane-chunk when a lane owns one 16-byte chunk of the row
#ifndef GNN_SPMM_U_NARROW
#define GNN_SPMM_U_NARROW 16
#endif
#ifndef GNN_SPMM_U_WIDE
#define GNN_SPMM_U_WIDE 8
#endif

#ifndef GNN_SPMM_RPG
#define GNN_SPMM_RPG 4
#endif
constexpr int kRowsPerGroup = GNN_SPMM_RPG;   // largest chunk: this many rows of the list per group
constexpr int kHubDegree = 1024;   // rows longer than this are split over the whole workgroup

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
    int32_t accumulate;
    int32_t rows_per_group;   // 1..kRowsPerGroup: rows of the list per LPR-lane group in one workgroup
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
    static __device__ __forceinline__ void store(void* p, int64_t off, const float (&v)[4], int n_valid, bool accumulate) {
        float* q = (float*)p + off;
        if (n_valid >= 4) {
            float4 o = make_float4(v[0], v[1], v[2], v[3]);
            if (accumulate) {
                float4 old = *(const float4*)q;
                o.x += old.x; o.y += old.y; o.z += old.z; o.w += old.w;
            }
            *(float4*)q = o;
        } else {
            for (int e = 0; e < n_valid; ++e) q[e] = accumulate ? q[e] + v[e] : v[e];
        }
    }
};

template <>
struct Elem<GNN_F32, 1> {
    static constexpr int VE = 1;
    using Raw = float;
    static __device__ __forceinline__ Raw load(const void* p, int64_t off) { return ((const float*)p)[off]; }
    static __device__ __forceinline__ void fma(float (&acc)[1], float w, const Raw& r) { acc[0] = fmaf(w, r, acc[0]); }
    static __device__ __forceinline__ void store(void* p, int64_t off, const float (&v)[1], int n_valid, bool accumulate) {
        float* q = (float*)p + off;
        if (n_valid >= 1) q[0] = accumulate ? q[0] + v[0] : v[0];
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
    static __device__ __forceinline__ void store(void* p, int64_t off, const float (&v)[8], int n_valid, bool accumulate) {
        uint16_t* q = (uint16_t*)p + off;
        if (n_valid >= 8) {
            float t[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) t[e] = v[e];
            if (accumulate) {
                uint4 old = *(const uint4*)q;
                t[0] += bf16lo(old.x); t[1] += bf16hi(old.x); t[2] += bf16lo(old.y); t[3] += bf16hi(old.y);
                t[4] += bf16lo(old.z); t[5] += bf16hi(old.z); t[6] += bf16lo(old.w); t[7] += bf16hi(old.w);
            }
            uint4 o;
            o.x = pack_bf16(t[0], t[1]); o.y = pack_bf16(t[2], t[3]);
            o.z = pack_bf16(t[4], t[5]); o.w = pack_bf16(t[6], t[7]);
            *(uint4*)q = o;
        } else {
            for (int e = 0; e < n_valid; ++e) q[e] = f32_to_bf16(accumulate ? bf16_to_f32(q[e]) + v[e] : v[e]);
        }
    }
};

template <>
struct Elem<GNN_BF16, 1> {
    static constexpr int VE = 1;
    using Raw = uint16_t;
    static __device__ __forceinline__ Raw load(const void* p, int64_t off) { return ((const uint16_t*)p)[off]; }
    static __device__ __forceinline__ void fma(float (&acc)[1], float w, const Raw& r) { acc[0] = fmaf(w, bf16_to_f32(r), acc[0]); }
    static __device__ __forceinline__ void store(void* p, int64_t off, const float (&v)[1], int n_valid, bool accumulate) {
        uint16_t* q = (uint16_t*)p + off;
        if (n_valid >= 1) q[0] = f32_to_bf16(accumulate ? bf16_to_f32(q[0]) + v[0] : v[0]);
    }
};

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
// (plus U broadcast loads of the neighbour scale) before the first multiply-add.
template <typename E, int LPR, int NCH, int U>
__device__ __forceinline__ void consume_tile(const SpmmArgs& a, int cnt, int cnt_max, int sub, const int64_t (&col_off)[NCH],
                                             const bool (&col_ok)[NCH], const int32_t* s_idx, float (&acc)[NCH][E::VE]) {
    for (int k = 0; k < cnt_max; k += U) {
        typename E::Raw x[U][NCH];
        float w[U];
#pragma unroll
        for (int j = 0; j < U; ++j) {
            w[j] = 1.f;
            if (k + j < cnt) {
                const int32_t u = s_idx[sub * LPR + k + j];
                if (a.nbr_scale) w[j] = a.nbr_scale[u];
                const int64_t base = (int64_t)u * a.ldx;
#pragma unroll
                for (int c = 0; c < NCH; ++c)
                    if (col_ok[c]) x[j][c] = E::load(a.X, base + col_off[c]);
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
//   phase 2  hub rows (longer than kHubDegree) are taken one at a time by ALL groups (group q takes
//            tiles q, q+NG, ...); the partial sums meet in LDS and are added in group order.
// Which group handles a row does not change the order of its additions: results are bit-reproducible.
// At least four workgroups per CU (six when a lane holds a single chunk and eight loads): the gather is
// latency-bound, so resident wavefronts matter more than a few registers.
template <int DT, int VE, int LPR, int NCH, int U, bool FILTER>
__global__ __launch_bounds__(256, (NCH == 1 && U <= 8) ? 6 : 4) void spmm_rows_kernel(SpmmArgs a) {
    using E = Elem<DT, VE>;
    constexpr int RPW = kWave / LPR;
    constexpr int NG = 4 * RPW;
    constexpr int RPB = NG * kRowsPerGroup;  // largest chunk, <= 128
    constexpr int W = LPR * NCH * VE;        // feature columns per workgroup (grid.y blocks cover F)
    __shared__ int32_t s_idx_all[4][kWave];
    __shared__ int32_t s_row_v[RPB], s_row_s[RPB], s_row_e[RPB], s_row_hub[RPB];
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
        const int32_t s = a.row_ptr[v], e = a.row_ptr[v + 1];
        const bool hub = e - s > kHubDegree;
        s_row_v[r] = v;
        s_row_s[r] = s;
        s_row_e[r] = hub ? s : e;
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
    if (FILTER) d_c = (have && pc + sl < ec) ? a.dist[u_c] : -1;
    while (__ballot(have) != 0ull) {  // uniform over the wave
        const bool row_done = have && pc + LPR >= ec;
        int jnn;
        int32_t pnn, enn;
        bool have_nn;
        advance(jn, pn, en, have_n, jnn, pnn, enn, have_nn);
        const int32_t u_nn = (have_nn && pnn + sl < enn) ? a.col_idx[pnn + sl] : 0;  // two tiles ahead
        int32_t d_n = 0;
        if (FILTER) d_n = (have_n && pn + sl < en) ? a.dist[u_n] : -1;               // one tile ahead

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
                        E::store(a.Y, (int64_t)v * a.ldy + col_off[c], o, rest >= VE ? VE : (int)rest, a.accumulate != 0);
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
        const int32_t hs = s_row_s[q], he = a.row_ptr[hv + 1];
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
            if (FILTER) d = sl < left ? a.dist[u] : -1;
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
                Elem<DT, 1>::store(a.Y, (int64_t)hv * a.ldy + gcol, o, 1, a.accumulate != 0);
            }
        }
        __syncthreads();
    }
}

template <int DT, int VE, int LPR, int NCH, bool FILTER>
static int32_t launch_rows(const SpmmArgs& a, hipStream_t stream) {
    constexpr int U = NCH == 1 ? (LPR < 64 ? GNN_SPMM_U_NARROW : GNN_SPMM_U_WIDE) : (NCH == 2 ? 4 : (NCH == 3 ? 3 : 2));
    constexpr int NG = 4 * (kWave / LPR);
    constexpr int W = LPR * NCH * VE;
    // chunk size: as large as possible (better balance inside a workgroup) while the launch still
    // has about 16 workgroups per CU
    SpmmArgs b = a;
    int rpg = (int)((int64_t)a.n_active / ((int64_t)NG * 4096));
    b.rows_per_group = rpg < 1 ? 1 : (rpg > kRowsPerGroup ? kRowsPerGroup : rpg);
    const int rpb = NG * b.rows_per_group;
    dim3 grid((unsigned)(((int64_t)a.n_active + rpb - 1) / rpb), (unsigned)((a.F + W - 1) / W));
    spmm_rows_kernel<DT, VE, LPR, NCH, U, FILTER><<<grid, 256, 0, stream>>>(b);
    GNN_LAUNCH_CHECK("spmm_rows_kernel");
    return GNN_OK;
}

template <int DT, bool FILTER>
static int32_t dispatch(const SpmmArgs& a, bool vec_ok, hipStream_t stream) {
    constexpr int VE = DT == GNN_F32 ? 4 : 8;
    const int F = a.F;
    // any alignment / leading dimension: element-wise lanes, 256 columns per workgroup
    if (!vec_ok) return launch_rows<DT, 1, 64, 4, FILTER>(a, stream);
    if (F <= 16 * VE) return launch_rows<DT, VE, 16, 1, FILTER>(a, stream);
    if (F <= 32 * VE) return launch_rows<DT, VE, 32, 1, FILTER>(a, stream);
    if (F <= 64 * VE) return launch_rows<DT, VE, 64, 1, FILTER>(a, stream);
    if (F <= 128 * VE) return launch_rows<DT, VE, 64, 2, FILTER>(a, stream);
    return launch_rows<DT, VE, 64, 3, FILTER>(a, stream);
}

static int32_t spmm_common(const gnn_csr* g, const char* gname, const int32_t* rows, int32_t n_active, const int32_t* dist,
                           int32_t max_dist, const void* X, int64_t ldx, void* Y, int64_t ldy, int32_t F, int32_t dtype,
                           const float* out_scale, const float* nbr_scale, int32_t accumulate, hipStream_t stream) {
    GNN_CHECK(check_csr(g, gname));
    GNN_REQUIRE(n_active >= 0, GNN_ERR_INVALID_ARG, "negative row count");
    GNN_REQUIRE(rows != nullptr || n_active <= g->n_rows, GNN_ERR_SHAPE, "n_active %d exceeds n_rows %d", n_active, g->n_rows);
    GNN_REQUIRE(dtype == GNN_F32 || dtype == GNN_BF16, GNN_ERR_UNSUPPORTED, "unknown dtype %d", dtype);
    GNN_REQUIRE(F >= 0, GNN_ERR_INVALID_ARG, "F < 0");
    GNN_REQUIRE(ldx >= F && ldy >= F, GNN_ERR_SHAPE, "leading dimension smaller than F = %d", F);
    if (n_active == 0 || F == 0) return GNN_OK;
    GNN_REQUIRE(X != nullptr && Y != nullptr, GNN_ERR_INVALID_ARG, "X or Y is NULL");

    SpmmArgs a;
    a.row_ptr = g->row_ptr; a.col_idx = g->col_idx; a.rows = rows; a.n_active = n_active;
    a.X = X; a.ldx = ldx; a.Y = Y; a.ldy = ldy; a.F = F;
    a.out_scale = out_scale; a.nbr_scale = nbr_scale; a.dist = dist; a.max_dist = max_dist;
    a.accumulate = accumulate;
    a.rows_per_group = 1;

    const int ve = dtype == GNN_F32 ? 4 : 8;
    const bool vec_ok = ((uintptr_t)X % 16 == 0) && ((uintptr_t)Y % 16 == 0) && ldx % ve == 0 && ldy % ve == 0;
    const bool filter = dist != nullptr;
    if (dtype == GNN_F32) return filter ? dispatch<GNN_F32, true>(a, vec_ok, stream) : dispatch<GNN_F32, false>(a, vec_ok, stream);
    return filter ? dispatch<GNN_BF16, true>(a, vec_ok, stream) : dispatch<GNN_BF16, false>(a, vec_ok, stream);
}

}  // namespace gnnhot

using namespace gnnhot;

extern "C" int32_t gnn_masked_spmm_fwd(const gnn_csr* g, const int32_t* rows, int32_t n_active, const void* X, int64_t ldx,
                                       void* Y, int64_t ldy, int32_t F, int32_t dtype, const float* row_scale,
                                       const float* col_scale, void* stream) {
    return spmm_common(g, "g", rows, n_active, nullptr, 0, X, ldx, Y, ldy, F, dtype, row_scale, col_scale, 0, (hipStream_t)stream);
}

extern "C" int32_t gnn_masked_spmm_bwd(const gnn_csr* gT, const int32_t* out_rows, int32_t n_out, const int32_t* dist,
                                       int32_t max_active_dist, const void* dY, int64_t lddy, void* dX, int64_t lddx, int32_t F,
                                       int32_t dtype, const float* row_scale, const float* col_scale, int32_t accumulate,
                                       void* stream) {
    GNN_REQUIRE(accumulate == 0 || accumulate == 1, GNN_ERR_INVALID_ARG, "accumulate must be 0 or 1");
    return spmm_common(gT, "gT", out_rows, n_out, dist, max_active_dist, dY, lddy, dX, lddx, F, dtype, col_scale, row_scale,
                       accumulate, (hipStream_t)stream);
}
