// A whole layer's forward pass in one kernel (paper section 2.1, both halves of the layer equation): the masked
// aggregation of a tile of rows is formed in LDS and fed straight to the MFMAs of the feature transform,
//     H[v] = act( (rs[v] * sum_{u in row(v)} cs[u] X[u]) W_neigh + X[v] W_self + b ),
// so the aggregate A_l is never written to (nor read back from) HBM.
//
// Mapping to CDNA4.  One workgroup (4 wavefronts) owns 64 consecutive entries of the row list.
//   phase A  gather: LPR lanes (8, 16 or 32: one 16-byte chunk each) span a row of X; the NG = 256 / LPR lane groups take
//            the tile's rows in rounds.  A group reads LPR neighbour ids (and scale factors) with one coalesced load, hands
//            them round by shuffle, and keeps eight row loads in flight per lane; loops run to the longest row of the
//            wavefront (predicated), so control flow stays uniform.  The sum is scaled, rounded to the storage type - exactly
//            where the two-call path rounds A_l - and written to the LDS tile, chunk c of row r at slot c ^ (r & 7)
//            (conflict-free 16-byte reads down a column of rows).  Rows longer than 512 entries are left to
//   phase A' hubs: all groups of the workgroup share one such row (group q takes id tiles q, q + NG, ...), the partial
//            sums meet in LDS and are added in group order.  Fixed order everywhere: bit-reproducible.
//   phase B  transform: wave (wm, wn) owns 32 rows x half of the output columns.  Its A operand comes from the LDS tile
//            (neighbour half) and directly from X in the MFMA operand layout (self half: lane (row, g) loads the 16 bytes
//            of chunk 2 kc + g of its row); the B operand comes from the transposed weights in the same layout - they are
//            at most 128 KB and stay in L2.  Four k-steps of loads are issued ahead of their MFMAs.
//   phase C  bias, activation, rounding; the tile is laid out row-major in LDS (over the aggregate) and leaves with
//            16-byte stores.
// Against the two-call path this saves one write and one read of A_l per layer; it pays with a gather phase that has no
// dynamic row claiming and shares its registers and LDS with the product (measured figures: see the repository's design
// notes).  The backward pass of a layer computed this way cannot use A_l: its weight gradient is H_{l-1}^T Agg^T(dZ).
#include "common.h"
#include <type_traits>

namespace gnnhot {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kFusedBM = 64;        // rows per workgroup
constexpr int kFusedHub = 512;      // longer rows are shared by the whole workgroup
constexpr int kFusedU = 8;          // row loads in flight per lane

struct FusedArgs {
    const int32_t* row_ptr;
    const int32_t* col_idx;
    const int32_t* rows;       // nullable
    int32_t n_active;
    const void* X;
    int64_t ldx;
    int32_t K;
    int32_t kp;                // K rounded up to a whole 32-byte k-step, in elements
    const float* out_scale;    // nullable
    const float* nbr_scale;    // nullable
    const void* Wt0;           // [N][kp] transposed W_neigh, columns K..kp zero
    const void* Wt1;           // nullable: the same for W_self
    const float* bias;         // nullable
    int32_t N;
    void* H;
    int64_t ldh;
    int32_t relu;
    int32_t h_vec;             // 16-byte stores to rows of H allowed
};

template <int DT>
__device__ __forceinline__ void fma_chunk(float (&acc)[16 / (DT == GNN_F32 ? 4 : 2)], float w, const u32x4& r) {
    if (DT == GNN_F32) {
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[t] = fmaf(w, __uint_as_float(r[t]), acc[t]);
    } else {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            acc[2 * t] = fmaf(w, bf16lo(r[t]), acc[2 * t]);
            acc[2 * t + 1] = fmaf(w, bf16hi(r[t]), acc[2 * t + 1]);
        }
    }
}

// VE floats -> one 16-byte chunk of the storage type; elements at or beyond n_valid become zero
template <int DT>
__device__ __forceinline__ u32x4 pack_chunk(const float* v, int n_valid) {
    u32x4 o;
    if (DT == GNN_F32) {
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = t < n_valid ? __float_as_uint(v[t]) : 0u;
    } else {
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = pack_bf16(2 * t < n_valid ? v[2 * t] : 0.f, 2 * t + 1 < n_valid ? v[2 * t + 1] : 0.f);
    }
    return o;
}

template <int DT>
__device__ __forceinline__ u32x4 keep_first(u32x4 r, int n_valid) {
    if (DT == GNN_F32) {
#pragma unroll
        for (int t = 0; t < 4; ++t) r[t] = n_valid > t ? r[t] : 0u;
    } else {
#pragma unroll
        for (int t = 0; t < 4; ++t) r[t] &= (n_valid > 2 * t ? 0xffffu : 0u) | (n_valid > 2 * t + 1 ? 0xffff0000u : 0u);
    }
    return r;
}

// LPR: lanes per gathered row (kp * ES / 16 chunks, rounded up to 8, 16 or 32).  NT: 32-column blocks per wave (the
// workgroup covers 64 * NT output columns).
template <int DT, int LPR, int NT>
__global__ __launch_bounds__(256) void fused_agg_linear_kernel(FusedArgs a) {
    constexpr int ES = DT == GNN_F32 ? 4 : 2, VE = 16 / ES;
    constexpr int RPW = kWave / LPR, NG = 4 * RPW, BM = kFusedBM, U = kFusedU;
    extern __shared__ __attribute__((aligned(16))) uint32_t smem[];
    const int chunks = a.kp / VE;                 // 16-byte chunks per row of the tile (8 .. 32)
    const int RW = (chunks + 7) / 8 * 8 * 4;      // words per tile row: whole groups of eight chunks (the slot swizzle stays inside one)
    constexpr int NCOL = 64 * NT;                 // output columns the workgroup computes
    constexpr int CW = NCOL * ES / 4 + 4;         // words per row of the staged output tile
    const int tile_words = BM * RW > BM * CW ? BM * RW : BM * CW;
    uint32_t* sAgg = smem;
    float* s_red = (float*)(smem + tile_words);   // [NG][LPR * VE] partial sums of a hub row
    int32_t* s_hub = (int32_t*)(s_red + NG * LPR * VE);   // [BM]
    int32_t* s_vid = s_hub + BM;                  // [BM] vertex id of every tile row (a valid one past the end)

    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane / LPR, sl = lane % LPR;
    const int gi = wave * RPW + sub;
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int n_tile = (int)((int64_t)a.n_active - m0 < BM ? (int64_t)a.n_active - m0 : BM);
    const bool col_ok = sl < chunks;              // this lane owns a chunk of the tile row
    const int my_valid = a.K - sl * VE;           // elements of that chunk that exist in X (<= 0: padding only, never loaded)
    const bool col_ld = my_valid > 0;

    if (tid < BM) {
        s_hub[tid] = 0;
        const int64_t m = tid < n_tile ? m0 + tid : m0;
        s_vid[tid] = a.rows ? a.rows[m] : (int32_t)m;
    }
    __syncthreads();

    // One id tile of a row: gather up to LPR neighbour rows, U at a time.  `cnt` may differ between the groups of a wave,
    // cnt_max is uniform.
    auto gather_tile = [&](int32_t u_mine, float w_mine, int cnt, int cnt_max, float (&acc)[VE]) {
        for (int k = 0; k < cnt_max; k += U) {
            u32x4 x[U];
            float w[U];
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const int32_t u = __shfl(u_mine, k + j, LPR);
                w[j] = __shfl(w_mine, k + j, LPR);
                if (k + j < cnt && col_ld) x[j] = *(const u32x4*)((const char*)a.X + ((int64_t)u * a.ldx + sl * VE) * ES);
            }
#pragma unroll
            for (int j = 0; j < U; ++j)
                if (k + j < cnt && col_ld) fma_chunk<DT>(acc, w[j], x[j]);
        }
    };
    auto store_row = [&](int r, const float (&acc)[VE], float sc) {
        if (!col_ok) return;
        float o[VE];
#pragma unroll
        for (int t = 0; t < VE; ++t) o[t] = acc[t] * sc;
        *(u32x4*)&sAgg[r * RW + ((sl ^ (r & 7)) << 2)] = pack_chunk<DT>(o, my_valid);
    };

    // ---- phase A
    for (int r0 = 0; r0 < BM; r0 += NG) {   // uniform over the workgroup
        const int r = r0 + gi;
        const bool have = r < n_tile;
        int32_t s = 0, e = 0;
        float sc = 0.f;
        bool hub = false;
        if (have) {
            const int32_t v = s_vid[r];
            s = a.row_ptr[v];
            e = a.row_ptr[v + 1];
            sc = a.out_scale ? a.out_scale[v] : 1.f;
            hub = e - s > kFusedHub;
            if (hub) {
                if (sl == 0) s_hub[r] = 1;
                e = s;
            }
        }
        float acc[VE];
#pragma unroll
        for (int t = 0; t < VE; ++t) acc[t] = 0.f;
        int len_max = e - s;
#pragma unroll
        for (int d = LPR; d < kWave; d <<= 1) len_max = max(len_max, __shfl_xor(len_max, d, kWave));
        for (int off = 0; off < len_max; off += LPR) {   // uniform over the wavefront
            const int32_t p = s + off + sl;
            const bool in = p < e;
            const int32_t u_mine = in ? a.col_idx[p] : 0;
            const float w_mine = (in && a.nbr_scale) ? a.nbr_scale[u_mine] : 1.f;
            int cnt = e - s - off;
            cnt = cnt < 0 ? 0 : (cnt < LPR ? cnt : LPR);
            int cnt_max = cnt;
#pragma unroll
            for (int d = LPR; d < kWave; d <<= 1) cnt_max = max(cnt_max, __shfl_xor(cnt_max, d, kWave));
            gather_tile(u_mine, w_mine, cnt, cnt_max, acc);
        }
        if (r < BM && !hub) store_row(r, acc, sc);   // rows past the end of the list are zero rows of the tile
    }
    __syncthreads();

    // ---- phase A': hub rows, one at a time, by all groups
    for (int r = 0; r < n_tile; ++r) {
        if (!s_hub[r]) continue;   // uniform over the workgroup
        const int32_t v = s_vid[r];
        const int32_t s = a.row_ptr[v], e = a.row_ptr[v + 1];
        float acc[VE];
#pragma unroll
        for (int t = 0; t < VE; ++t) acc[t] = 0.f;
        for (int32_t base = s; base < e; base += NG * LPR) {   // uniform over the workgroup
            const int32_t p0 = base + gi * LPR;
            const int32_t p = p0 + sl;
            const bool in = p < e;
            const int32_t u_mine = in ? a.col_idx[p] : 0;
            const float w_mine = (in && a.nbr_scale) ? a.nbr_scale[u_mine] : 1.f;
            int cnt = e - p0;
            cnt = cnt < 0 ? 0 : (cnt < LPR ? cnt : LPR);
            int cnt_max = cnt;
#pragma unroll
            for (int d = LPR; d < kWave; d <<= 1) cnt_max = max(cnt_max, __shfl_xor(cnt_max, d, kWave));
            gather_tile(u_mine, w_mine, cnt, cnt_max, acc);
        }
#pragma unroll
        for (int t = 0; t < VE; ++t) s_red[gi * (LPR * VE) + sl * VE + t] = acc[t];
        __syncthreads();
        const float sc = a.out_scale ? a.out_scale[v] : 1.f;
        for (int c = tid; c < chunks; c += 256) {
            float o[VE];
#pragma unroll
            for (int t = 0; t < VE; ++t) {
                float sum = 0.f;
                for (int q = 0; q < NG; ++q) sum += s_red[q * (LPR * VE) + c * VE + t];
                o[t] = sum * sc;
            }
            *(u32x4*)&sAgg[r * RW + ((c ^ (r & 7)) << 2)] = pack_chunk<DT>(o, a.K - c * VE);
        }
        __syncthreads();
    }

    // ---- phase B
    const int wm = wave & 1, wn = wave >> 1;
    const int li = lane & 31, g = lane >> 5;
    const int trow = wm * 32 + li;                        // tile row this lane feeds
    const char* x_self = (const char*)a.X + (int64_t)s_vid[trow] * a.ldx * ES;
    v16f acc[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    int64_t wt_off[NT];                                   // byte offset of this lane's row of the transposed weights, per column block
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int n = (wn * NT + j) * 32 + li;
        wt_off[j] = (int64_t)(n < a.N ? n : 0) * a.kp * ES;
    }
    auto mma = [&](v16f& c, const u32x4& x, const u32x4& y) {
        if (DT == GNN_F32) {
#pragma unroll
            for (int t = 0; t < 4; ++t) c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(x[t]), __uint_as_float(y[t]), c, 0, 0, 0);
        } else {
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, x), __builtin_bit_cast(v8bf, y), c, 0, 0, 0);
        }
    };
    const int k_steps = chunks / 2;                       // 32 bytes of the reduction per step: chunk 2 kc + g for half g
    constexpr int KU = NT == 4 ? 2 : 4;                   // steps whose loads are issued ahead of their MFMAs
    // One source (SELF false: the aggregate in LDS, true: the vertex's own row in X) against its transposed weights.
    // Straight-line code per source: the accumulators stay in place between the two.
    auto run_source = [&](auto self_tag, const char* wt) {
        constexpr bool SELF = decltype(self_tag)::value;
        for (int kc0 = 0; kc0 < k_steps; kc0 += KU) {
            u32x4 fa[KU], fb[KU][NT];
#pragma unroll
            for (int q = 0; q < KU; ++q) {
                const int kc = kc0 + q < k_steps ? kc0 + q : k_steps - 1;   // a repeat past the end: loaded, not multiplied
                const int c = kc * 2 + g;
                if (!SELF) fa[q] = *(const u32x4*)&sAgg[trow * RW + ((c ^ (trow & 7)) << 2)];
                else fa[q] = keep_first<DT>(*(const u32x4*)(x_self + (int64_t)(a.K - c * VE > 0 ? c : 0) * 16), a.K - c * VE);
#pragma unroll
                for (int j = 0; j < NT; ++j) fb[q][j] = *(const u32x4*)(wt + wt_off[j] + (int64_t)c * 16);
            }
#pragma unroll
            for (int q = 0; q < KU; ++q) {
                if (kc0 + q < k_steps) {
#pragma unroll
                    for (int j = 0; j < NT; ++j) mma(acc[j], fa[q], fb[q][j]);
                }
            }
        }
    };
    run_source(std::false_type{}, (const char*)a.Wt0);
    if (a.Wt1 != nullptr) run_source(std::true_type{}, (const char*)a.Wt1);   // uniform over the grid
    __syncthreads();   // every wave has read the aggregate: the tile is free for the output

    // ---- phase C: acc[j][r] is H[row (r/4)*8 + g*4 + r%4][column li] of its 32 x 32 block
    uint32_t* sC = smem;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int col = (wn * NT + j) * 32 + li;
        const float bv = (a.bias && col < a.N) ? a.bias[col] : 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = wm * 32 + (r >> 2) * 8 + g * 4 + (r & 3);
            float v = acc[j][r] + bv;
            if (a.relu) v = v > 0.f ? v : 0.f;
            if (DT == GNN_F32) sC[row * CW + col] = __float_as_uint(v);
            else ((uint16_t*)sC)[row * (CW * 2) + col] = f32_to_bf16(v);
        }
    }
    __syncthreads();
    constexpr int CPR = NCOL / VE;   // 16-byte chunks per staged row
    for (int idx = tid; idx < BM * CPR; idx += 256) {
        const int row = idx / CPR, ch = idx % CPR;
        const int n = ch * VE;
        if (row >= n_tile || n >= a.N) continue;
        const u32x4 v = *(const u32x4*)&sC[row * CW + ch * 4];
        char* dst = (char*)a.H + ((int64_t)s_vid[row] * a.ldh + n) * ES;
        if (n + VE <= a.N && a.h_vec) {
            *(u32x4*)dst = v;
        } else {
            for (int t = 0; t < VE && n + t < a.N; ++t) {
                if (DT == GNN_F32) ((uint32_t*)dst)[t] = v[t];
                else ((uint16_t*)dst)[t] = (uint16_t)(v[t >> 1] >> ((t & 1) * 16));
            }
        }
    }
}

// Wt[n][0:kp] = W[0:K][n] followed by zeros (the reduction is padded to whole 32-byte steps: padding must multiply as zero)
template <int DT>
__global__ __launch_bounds__(256) void fused_transpose_kernel(const void* __restrict__ W, int32_t K, int32_t N, int32_t kp,
                                                              void* __restrict__ Wt) {
    const int64_t total = (int64_t)N * kp;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int32_t n = (int32_t)(t / kp), k = (int32_t)(t % kp);
        if (DT == GNN_F32) ((float*)Wt)[t] = k < K ? ((const float*)W)[(int64_t)k * N + n] : 0.f;
        else ((uint16_t*)Wt)[t] = k < K ? ((const uint16_t*)W)[(int64_t)k * N + n] : (uint16_t)0;
    }
}

template <int DT, int LPR>
static int32_t launch_fused(const FusedArgs& a, hipStream_t stream) {
    constexpr int ES = DT == GNN_F32 ? 4 : 2, VE = 16 / ES;
    const int nt = a.N <= 64 ? 1 : (a.N <= 128 ? 2 : 4);
    const int rw = (a.kp / VE + 7) / 8 * 8 * 4, cw = 64 * nt * ES / 4 + 4;
    const size_t tile_words = (size_t)kFusedBM * (rw > cw ? rw : cw);
    const size_t lds = tile_words * 4 + (size_t)256 * VE * 4 + 2 * kFusedBM * 4;
    const unsigned grid = (unsigned)(((int64_t)a.n_active + kFusedBM - 1) / kFusedBM);
    if (nt == 1) fused_agg_linear_kernel<DT, LPR, 1><<<grid, 256, lds, stream>>>(a);
    else if (nt == 2) fused_agg_linear_kernel<DT, LPR, 2><<<grid, 256, lds, stream>>>(a);
    else fused_agg_linear_kernel<DT, LPR, 4><<<grid, 256, lds, stream>>>(a);
    GNN_LAUNCH_CHECK("fused_agg_linear_kernel");
    return GNN_OK;
}

template <int DT>
static int32_t run_fused(FusedArgs a, const void* Wn, const void* Ws, void* Wt0, void* Wt1, hipStream_t stream) {
    constexpr int ES = DT == GNN_F32 ? 4 : 2, VE = 16 / ES;
    const int grid = grid_for((int64_t)a.N * a.kp, 256, 1024);
    fused_transpose_kernel<DT><<<grid, 256, 0, stream>>>(Wn, a.K, a.N, a.kp, Wt0);
    GNN_LAUNCH_CHECK("fused_transpose_kernel");
    if (Ws) {
        fused_transpose_kernel<DT><<<grid, 256, 0, stream>>>(Ws, a.K, a.N, a.kp, Wt1);
        GNN_LAUNCH_CHECK("fused_transpose_kernel");
    }
    a.Wt0 = Wt0;
    a.Wt1 = Ws ? Wt1 : nullptr;
    const int chunks = a.kp / VE;
    if (chunks <= 8) return launch_fused<DT, 8>(a, stream);
    if (chunks <= 16) return launch_fused<DT, 16>(a, stream);
    return launch_fused<DT, 32>(a, stream);
}

}  // namespace gnnhot

using namespace gnnhot;

extern "C" int32_t gnn_fused_layer_fwd(const gnn_csr* g, const int32_t* rows, int32_t n_active, const void* X, int64_t ldx, int32_t K,
                                       const float* row_scale, const float* col_scale, const void* W_neigh, const void* W_self,
                                       const float* bias, int32_t N, void* H_out, int64_t ld_out, int32_t relu, int32_t dtype,
                                       void* ws, size_t* ws_bytes, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    GNN_CHECK(check_csr(g, "g"));
    GNN_REQUIRE(n_active >= 0, GNN_ERR_INVALID_ARG, "negative row count");
    GNN_REQUIRE(rows != nullptr || n_active <= g->n_rows, GNN_ERR_SHAPE, "n_active %d exceeds n_rows %d", n_active, g->n_rows);
    GNN_REQUIRE(dtype == GNN_F32 || dtype == GNN_BF16, GNN_ERR_UNSUPPORTED, "unknown dtype %d", dtype);
    GNN_REQUIRE(K >= 1 && N >= 1, GNN_ERR_INVALID_ARG, "K and N must be positive");
    GNN_REQUIRE(ldx >= K && ld_out >= N, GNN_ERR_SHAPE, "leading dimension smaller than the width");
    GNN_REQUIRE(relu == 0 || relu == 1, GNN_ERR_INVALID_ARG, "relu must be 0 or 1");
    GNN_REQUIRE(g->edge_keep == nullptr, GNN_ERR_UNSUPPORTED, "per-layer edge masks are known to gnn_masked_spmm_fwd only");
    const int es = dtype == GNN_F32 ? 4 : 2;
    const int32_t kp = (int32_t)align_up((size_t)K, (size_t)(32 / es));
    // the aggregate of 64 rows and the output tile live in LDS: rows of 128 to 512 bytes in, at most 512 bytes out
    GNN_REQUIRE((int64_t)kp * es >= 128 && (int64_t)kp * es <= 512 && (int64_t)N * es <= 512, GNN_ERR_UNSUPPORTED,
                "the fused layer takes input rows of 128 to 512 bytes and output rows of at most 512 bytes "
                "(K = %d, N = %d, %d-byte elements): use gnn_masked_spmm_fwd + gnn_linear_fwd", K, N, es);
    GNN_REQUIRE(((uintptr_t)X % 16 == 0) && (ldx * es) % 16 == 0, GNN_ERR_UNSUPPORTED, "X rows must be 16-byte aligned");
    WsCarver carve(ws);
    char* Wt0 = carve.take<char>((size_t)N * kp * es);
    char* Wt1 = carve.take<char>((size_t)N * kp * es);
    bool query;
    GNN_CHECK(ws_protocol(ws, ws_bytes, carve.used, &query));
    if (query) return GNN_OK;
    if (n_active == 0) return GNN_OK;
    GNN_REQUIRE(X && W_neigh && H_out, GNN_ERR_INVALID_ARG, "X, W_neigh or H_out is NULL");
    FusedArgs a;
    a.row_ptr = g->row_ptr; a.col_idx = g->col_idx; a.rows = rows; a.n_active = n_active;
    a.X = X; a.ldx = ldx; a.K = K; a.kp = kp; a.out_scale = row_scale; a.nbr_scale = col_scale;
    a.Wt0 = nullptr; a.Wt1 = nullptr; a.bias = bias; a.N = N; a.H = H_out; a.ldh = ld_out; a.relu = relu;
    a.h_vec = ((uintptr_t)H_out % 16 == 0) && (ld_out * es) % 16 == 0;
    if (dtype == GNN_F32) return run_fused<GNN_F32>(a, W_neigh, W_self, Wt0, Wt1, stream);
    return run_fused<GNN_BF16>(a, W_neigh, W_self, Wt0, Wt1, stream);
}
