// Dense feature transform of a GNN layer and its backward pass (paper section 2.1: the
// aggregated vector, optionally combined with the vertex's own previous vector, is
// multiplied by the layer's weights and passed through the activation).
//
// Two MFMA GEMM kernels for gfx950 carry all of it:
//   gemm_nt   C[m, n] = epilogue( sum_src sum_k A_src[row(m), k] * Bt_src[n, k] )
//             forward  (Bt = W^T, made once per call in the workspace; bias + ReLU epilogue)
//             dA / dX_self = dZ W^T  (Bt = W as stored; rows scattered back through `rows`)
//   gemm_tn   P[split][k, n] = sum_{m in split} A_src[row(m), k] * D[m, n]
//             dW_neigh / dW_self = A^T dZ, reduced over fixed row splits, then summed in
//             split order by reduce_partials (deterministic, no atomics).
// fp32 uses v_mfma_f32_32x32x2_f32, bf16 uses v_mfma_f32_32x32x16_bf16 (fp32 accumulate).
//
// Tiling.  256 threads = 4 wavefronts per workgroup; every LDS tile row is 128 bytes of the
// reduction (gemm_nt) so one global row read is a full cache line, padded to 144 bytes so
// that 16-byte LDS reads of 32 consecutive rows are conflict-free.  The reduction index of a
// tile is permuted between the two halves of the wavefront (half g owns elements
// [g*BK/2, (g+1)*BK/2)) so that each lane fetches its whole operand strip with four
// ds_read_b128; both operands use the same permutation, which leaves the product unchanged.
// The next tile is prefetched into registers while the current one feeds the MFMAs.
// Workgroup ids are remapped so that consecutive tiles share an XCD (and its L2).
#include "common.h"
#include <mutex>

namespace gnnhot {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef short v4s __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));

// ds_read_b64_tr_b16: every lane hands in the LDS address of four 16-bit elements; within each group of 16 lanes
// the 16 x 4 block is transposed (lane j receives element j%4 of the lanes 4e + j/4, e = 0..3).
__device__ __forceinline__ v4s lds_tr16(const uint16_t* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4s __attribute__((address_space(3)))*)p);
}

#ifndef GNN_NT_PF_BF16
#define GNN_NT_PF_BF16 2
#endif
#ifndef GNN_NT_PF_F32
#define GNN_NT_PF_F32 1
#endif
#ifndef GNN_NT_MINB_NARROW
#define GNN_NT_MINB_NARROW 3
#endif
#ifndef GNN_NT_MINB
#define GNN_NT_MINB 3
#endif

constexpr int kMaxDim = 4096;
constexpr int kLdsRowWords = 36;  // 128 B of data + 16 B pad

template <int DT>
struct DTy {
    static constexpr int ES = DT == GNN_F32 ? 4 : 2;  // bytes per element
    static constexpr int EPV = 16 / ES;               // elements per 16-byte vector
};

// 16 bytes from row-major storage with element-granular bounds; `n_valid` elements from
// `p` are in range (<= 0: none).  Falls back to element loads at a ragged edge or when the
// address is not 16-byte aligned.
template <int DT>
__device__ __forceinline__ uint4 load16(const void* base, int64_t elem_off, int n_valid, bool vec_ok) {
    constexpr int EPV = DTy<DT>::EPV;
    uint4 r = make_uint4(0u, 0u, 0u, 0u);
    if (n_valid <= 0) return r;
    if (n_valid >= EPV && vec_ok) {
        if (DT == GNN_F32) return *(const uint4*)((const float*)base + elem_off);
        return *(const uint4*)((const uint16_t*)base + elem_off);
    }
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    if (DT == GNN_F32) {
        const uint32_t* p = (const uint32_t*)base + elem_off;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (e < n_valid) w[e] = p[e];
    } else {
        const uint16_t* p = (const uint16_t*)base + elem_off;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (e < n_valid) w[e >> 1] |= (uint32_t)p[e] << ((e & 1) * 16);
    }
    return make_uint4(w[0], w[1], w[2], w[3]);
}

// Fast path used when every row of the operand is 16-byte aligned and its leading dimension is a
// multiple of the vector.  load_raw issues ONE unconditional 16-byte load (an out-of-range chunk reads
// element 0 of the matrix instead, which is always addressable), so a whole tile's loads form a
// straight line that can stay in flight across the MFMAs; fix_chunk, applied when the data is moved
// to LDS, zeroes what was out of range and, on a ragged last tile, the elements at or beyond
// n_valid, so padding can never reach the MFMAs.
template <int DT>
__device__ __forceinline__ uint4 load_raw(const void* base, int64_t elem_off, bool in_range) {
    const int64_t off = in_range ? elem_off : 0;
    if (DT == GNN_F32) return *(const uint4*)((const float*)base + off);
    return *(const uint4*)((const uint16_t*)base + off);
}

template <int DT>
__device__ __forceinline__ uint4 fix_chunk(uint4 r, int n_valid) {
    if (DT == GNN_F32) {
        r.x = n_valid > 0 ? r.x : 0u;
        r.y = n_valid > 1 ? r.y : 0u;
        r.z = n_valid > 2 ? r.z : 0u;
        r.w = n_valid > 3 ? r.w : 0u;
    } else {
        r.x &= (n_valid > 0 ? 0xffffu : 0u) | (n_valid > 1 ? 0xffff0000u : 0u);
        r.y &= (n_valid > 2 ? 0xffffu : 0u) | (n_valid > 3 ? 0xffff0000u : 0u);
        r.z &= (n_valid > 4 ? 0xffffu : 0u) | (n_valid > 5 ? 0xffff0000u : 0u);
        r.w &= (n_valid > 6 ? 0xffffu : 0u) | (n_valid > 7 ? 0xffff0000u : 0u);
    }
    return r;
}

template <int DT>
__device__ __forceinline__ void store_elem(void* base, int64_t off, float v) {
    if (DT == GNN_F32) ((float*)base)[off] = v;
    else ((uint16_t*)base)[off] = f32_to_bf16(v);
}

template <int DT>
__device__ __forceinline__ float load_elem(const void* base, int64_t off) {
    if (DT == GNN_F32) return ((const float*)base)[off];
    return bf16_to_f32(((const uint16_t*)base)[off]);
}

// Workgroup id -> logical tile so that consecutive logical tiles run on the same XCD
// (ids are dealt round-robin over the 8 XCDs).  Grid must be 8 * ceil(total / 8).
__device__ __forceinline__ int64_t xcd_remap(int64_t id, int64_t total) {
    const int64_t per = (total + 7) / 8;
    return (id % 8) * per + id / 8;
}

// ------------------------------------------------------------------------------------------
// gemm_nt
// ------------------------------------------------------------------------------------------
struct GemmNT {
    const void* A[2];
    const void* Bt[2];
    int32_t n_src;
    int64_t lda, ldb;
    int32_t a_vec, b_vec;      // 16-byte loads allowed
    const int32_t* a_rows;     // nullable
    const int32_t* c_rows;     // nullable
    int32_t M, N, K;
    const float* bias;         // nullable
    int32_t relu;
    void* C;
    int64_t ldc;
    int32_t c_vec;             // 16-byte stores to C rows allowed
    // input gradient of a layer in the exchanged order: what is stored is (product + what C held, for the first n_acc
    // rows) where mask > 0, else 0.  mask: nullable, same rows and columns as C
    const void* mask;
    int64_t ldm;
    int32_t m_vec;             // 16-byte loads from mask rows allowed
    int32_t n_acc;
    int32_t M1;                // n_src == 2: only the rows m < M1 have a second source (INT32_MAX: all of them)
};

// The post-processing of that input gradient on one stored 16-byte vector / one element.
template <int DT>
__device__ __forceinline__ uint4 post_vec(uint4 v, const void* C, int64_t coff, bool acc, const void* mask, int64_t moff) {
    if (DT == GNN_F32) {
        float x[4] = {__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
        if (acc) {
            const float4 o = *(const float4*)((const float*)C + coff);
            x[0] += o.x; x[1] += o.y; x[2] += o.z; x[3] += o.w;
        }
        const float4 h = *(const float4*)((const float*)mask + moff);
        return make_uint4(__float_as_uint(h.x > 0.f ? x[0] : 0.f), __float_as_uint(h.y > 0.f ? x[1] : 0.f),
                          __float_as_uint(h.z > 0.f ? x[2] : 0.f), __float_as_uint(h.w > 0.f ? x[3] : 0.f));
    }
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    float x[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        x[2 * e] = bf16lo(w[e]);
        x[2 * e + 1] = bf16hi(w[e]);
    }
    if (acc) {
        const uint4 o4 = *(const uint4*)((const uint16_t*)C + coff);
        const uint32_t o[4] = {o4.x, o4.y, o4.z, o4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[2 * e] += bf16lo(o[e]);
            x[2 * e + 1] += bf16hi(o[e]);
        }
    }
    const uint4 h4 = *(const uint4*)((const uint16_t*)mask + moff);
    const uint32_t h[4] = {h4.x, h4.y, h4.z, h4.w};
    uint32_t r[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) r[e] = pack_bf16(bf16lo(h[e]) > 0.f ? x[2 * e] : 0.f, bf16hi(h[e]) > 0.f ? x[2 * e + 1] : 0.f);
    return make_uint4(r[0], r[1], r[2], r[3]);
}

template <int DT>
__device__ __forceinline__ float post_elem(float v, const void* C, int64_t coff, bool acc, const void* mask, int64_t moff) {
    float h;
    if (DT == GNN_F32) {
        if (acc) v += ((const float*)C)[coff];
        h = ((const float*)mask)[moff];
    } else {
        if (acc) v += bf16_to_f32(((const uint16_t*)C)[coff]);
        h = bf16_to_f32(((const uint16_t*)mask)[moff]);
    }
    return h > 0.f ? v : 0.f;
}

// post_vec with its two loads already done: v + old (where has_old) where h > 0, else 0.
template <int DT>
__device__ __forceinline__ uint4 post_apply(uint4 v, uint4 old, bool has_old, uint4 h4) {
    if (DT == GNN_F32) {
        float x[4] = {__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
        if (has_old) {
            x[0] += __uint_as_float(old.x); x[1] += __uint_as_float(old.y); x[2] += __uint_as_float(old.z); x[3] += __uint_as_float(old.w);
        }
        return make_uint4(__float_as_uint(__uint_as_float(h4.x) > 0.f ? x[0] : 0.f), __float_as_uint(__uint_as_float(h4.y) > 0.f ? x[1] : 0.f),
                          __float_as_uint(__uint_as_float(h4.z) > 0.f ? x[2] : 0.f), __float_as_uint(__uint_as_float(h4.w) > 0.f ? x[3] : 0.f));
    }
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    const uint32_t o[4] = {old.x, old.y, old.z, old.w};
    const uint32_t h[4] = {h4.x, h4.y, h4.z, h4.w};
    uint32_t r[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float lo = bf16lo(w[e]), hi = bf16hi(w[e]);
        if (has_old) {
            lo += bf16lo(o[e]);
            hi += bf16hi(o[e]);
        }
        r[e] = pack_bf16(bf16lo(h[e]) > 0.f ? lo : 0.f, bf16hi(h[e]) > 0.f ? hi : 0.f);
    }
    return make_uint4(r[0], r[1], r[2], r[3]);
}

template <int DT, int BN, int WM, int WN, bool VEC>
__global__ __launch_bounds__(256, BN == 128 ? GNN_NT_MINB : GNN_NT_MINB_NARROW) void gemm_nt_kernel(GemmNT a) {
    constexpr int BM = 128;
    constexpr int EPV = DTy<DT>::EPV;
    constexpr int BK = 8 * EPV;  // elements per 128-byte tile row
    constexpr int WTM = BM / WM, WTN = BN / WN, MT = WTM / 32, NT = WTN / 32;
    constexpr int A_CH = BM / 32, B_CH = BN / 32;  // 16-byte chunks per thread
    static_assert(WM * WN == 4 && MT >= 1 && NT >= 1, "bad wave layout");
    constexpr int PF = DT == GNN_BF16 ? GNN_NT_PF_BF16 : GNN_NT_PF_F32;  // register prefetch depth (bf16 steps are too short to hide a load)
    __shared__ __attribute__((aligned(16))) uint32_t smem[(BM + BN) * kLdsRowWords];
    uint32_t* sA = smem;
    uint32_t* sB = smem + BM * kLdsRowWords;

    const int tiles_n = (a.N + BN - 1) / BN, tiles_m = (a.M + BM - 1) / BM;
    const int64_t total = (int64_t)tiles_m * tiles_n;
    const int64_t tile = xcd_remap(blockIdx.x, total);
    if (tile >= total) return;
    const int m0 = (int)(tile / tiles_n) * BM, n0 = (int)(tile % tiles_n) * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, g = lane >> 5;
    const int ld_row = tid >> 3, ld_kc = tid & 7;  // loader: row within a 32-row band, 16-byte column

    int64_t a_off[A_CH];
    bool a_ok[A_CH];
#pragma unroll
    for (int c = 0; c < A_CH; ++c) {
        const int m = m0 + ld_row + 32 * c;
        a_ok[c] = m < a.M;
        const int64_t r = a_ok[c] ? (a.a_rows ? (int64_t)a.a_rows[m] : (int64_t)m) : 0;
        a_off[c] = r * a.lda;
    }
    int64_t b_off[B_CH];
    bool b_ok[B_CH];
#pragma unroll
    for (int c = 0; c < B_CH; ++c) {
        const int n = n0 + ld_row + 32 * c;
        b_ok[c] = n < a.N;
        b_off[c] = (int64_t)(b_ok[c] ? n : 0) * a.ldb;
    }

    v16f acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int k_tiles = (a.K + BK - 1) / BK;
    const int n_steps = k_tiles * ((a.n_src == 2 && m0 >= a.M1) ? 1 : a.n_src);   // a tile past M1 has one source only
    uint4 ra0[A_CH], rb0[B_CH], ra1[A_CH], rb1[B_CH];

    auto fetch = [&](int step, uint4 (&ra)[A_CH], uint4 (&rb)[B_CH]) {
        const int src = step / k_tiles;
        const int ke = (step % k_tiles) * BK + ld_kc * EPV;
        const int nv = a.K - ke;
        const void* Ab = a.A[src];
        const void* Bb = a.Bt[src];
        if (VEC) {
#pragma unroll
            for (int c = 0; c < A_CH; ++c) ra[c] = load_raw<DT>(Ab, a_off[c] + ke, a_ok[c] && nv > 0);
#pragma unroll
            for (int c = 0; c < B_CH; ++c) rb[c] = load_raw<DT>(Bb, b_off[c] + ke, b_ok[c] && nv > 0);
        } else {
#pragma unroll
            for (int c = 0; c < A_CH; ++c) ra[c] = load16<DT>(Ab, a_off[c] + ke, a_ok[c] ? nv : 0, a.a_vec != 0);
#pragma unroll
            for (int c = 0; c < B_CH; ++c) rb[c] = load16<DT>(Bb, b_off[c] + ke, b_ok[c] ? nv : 0, a.b_vec != 0);
        }
    };
    // edge: this workgroup's tile touches the end of M or N, or K is not a multiple of the tile row (uniform)
    const bool edge = m0 + BM > a.M || n0 + BN > a.N || a.K % BK != 0;
    auto stash = [&](int step, uint4 (&ra)[A_CH], uint4 (&rb)[B_CH]) {
        if (VEC && edge) {
            const int nv = a.K - ((step % k_tiles) * BK + ld_kc * EPV);
#pragma unroll
            for (int c = 0; c < A_CH; ++c) ra[c] = fix_chunk<DT>(ra[c], a_ok[c] ? nv : 0);
#pragma unroll
            for (int c = 0; c < B_CH; ++c) rb[c] = fix_chunk<DT>(rb[c], b_ok[c] ? nv : 0);
        }
        if (step >= k_tiles) {   // second source: rows at or past M1 contribute nothing
#pragma unroll
            for (int c = 0; c < A_CH; ++c)
                if (m0 + ld_row + 32 * c >= a.M1) ra[c] = make_uint4(0u, 0u, 0u, 0u);
        }
#pragma unroll
        for (int c = 0; c < A_CH; ++c) *(uint4*)&sA[(ld_row + 32 * c) * kLdsRowWords + ld_kc * 4] = ra[c];
#pragma unroll
        for (int c = 0; c < B_CH; ++c) *(uint4*)&sB[(ld_row + 32 * c) * kLdsRowWords + ld_kc * 4] = rb[c];
    };
    auto compute = [&]() {
        uint4 fa[MT][4], fb[NT][4];
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                fa[i][q] = *(const uint4*)&sA[(wm * WTM + i * 32 + li) * kLdsRowWords + g * 16 + q * 4];
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                fb[j][q] = *(const uint4*)&sB[(wn * WTN + j * 32 + li) * kLdsRowWords + g * 16 + q * 4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (DT == GNN_F32) {
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int i = 0; i < MT; ++i)
#pragma unroll
                        for (int j = 0; j < NT; ++j) {
                            const uint32_t av = t == 0 ? fa[i][q].x : (t == 1 ? fa[i][q].y : (t == 2 ? fa[i][q].z : fa[i][q].w));
                            const uint32_t bv = t == 0 ? fb[j][q].x : (t == 1 ? fb[j][q].y : (t == 2 ? fb[j][q].z : fb[j][q].w));
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(av), __uint_as_float(bv), acc[i][j], 0, 0, 0);
                        }
            } else {
#pragma unroll
                for (int i = 0; i < MT; ++i)
#pragma unroll
                    for (int j = 0; j < NT; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, fa[i][q]),
                                                                             __builtin_bit_cast(v8bf, fb[j][q]), acc[i][j], 0, 0, 0);
            }
        }
    };

    // Pipeline: LDS holds step s; register set (s+1)%2 holds step s+1 and, with PF == 2, the other set
    // is refilled with step s+2 before the MFMAs of step s start, so two tile loads overlap.
    if (n_steps > 0) fetch(0, ra0, rb0);
    if (PF == 2 && n_steps > 1) fetch(1, ra1, rb1);
    if (n_steps > 0) stash(0, ra0, rb0);
    __syncthreads();
    for (int step = 0; step < n_steps; step += 2) {
        if (PF == 2) {
            if (step + 2 < n_steps) fetch(step + 2, ra0, rb0);
        } else {
            if (step + 1 < n_steps) fetch(step + 1, ra1, rb1);
        }
        compute();
        __syncthreads();
        if (step + 1 < n_steps) {
            stash(step + 1, ra1, rb1);
            __syncthreads();
            if (PF == 2) {
                if (step + 3 < n_steps) fetch(step + 3, ra1, rb1);
            } else {
                if (step + 2 < n_steps) fetch(step + 2, ra0, rb0);
            }
            compute();
            __syncthreads();
            if (step + 2 < n_steps) {
                stash(step + 2, ra0, rb0);
                __syncthreads();
            }
        }
    }

    if (DT == GNN_BF16) {
        // bf16 epilogue through LDS: the accumulator layout gives 2-byte column-strided stores, so the
        // tile is first laid out row-major in LDS (bias + ReLU + rounding applied) and then written
        // with 16-byte stores, one 256-byte row segment per 16 lanes.
        constexpr int RS = BN / 2 + 4;  // words per LDS row of the C tile
        static_assert(BM * RS <= (BM + BN) * kLdsRowWords, "C tile does not fit the operand buffers");
        uint16_t* sC = (uint16_t*)smem;
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = wm * WTM + i * 32 + (r >> 2) * 8 + g * 4 + (r & 3);
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    const int col = wn * WTN + j * 32 + li;
                    float v = acc[i][j][r];
                    if (a.bias && n0 + col < a.N) v += a.bias[n0 + col];
                    if (a.relu) v = v > 0.f ? v : 0.f;
                    sC[row * (RS * 2) + col] = f32_to_bf16(v);
                }
            }
        __syncthreads();
        constexpr int CPR = BN / 8;  // 16-byte chunks per tile row
#pragma unroll
        for (int k = 0; k < BM * CPR / 256; ++k) {
            const int idx = tid + 256 * k;
            const int row = idx / CPR, ch = idx % CPR;
            const int m = m0 + row, n = n0 + ch * 8;
            if (m < a.M && n < a.N) {
                const int64_t crow = a.c_rows ? (int64_t)a.c_rows[m] : (int64_t)m;
                uint4 v = *(const uint4*)&smem[row * RS + ch * 4];
                uint16_t* dst = (uint16_t*)a.C + crow * a.ldc + n;
                if (n + 8 <= a.N && a.c_vec && (!a.mask || a.m_vec)) {
                    if (a.mask) v = post_vec<DT>(v, a.C, crow * a.ldc + n, m < a.n_acc, a.mask, crow * a.ldm + n);
                    *(uint4*)dst = v;
                } else {
                    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
                    for (int e = 0; e < 8 && n + e < a.N; ++e) {
                        uint16_t o = (uint16_t)(w[e >> 1] >> ((e & 1) * 16));
                        if (a.mask) o = f32_to_bf16(post_elem<DT>(bf16_to_f32(o), a.C, crow * a.ldc + n + e, m < a.n_acc, a.mask, crow * a.ldm + n + e));
                        dst[e] = o;
                    }
                }
            }
        }
        return;
    }

    // epilogue: acc[i][j][r] is C[row = (r/4)*8 + g*4 + r%4][col = li] of its 32x32 block
#pragma unroll
    for (int i = 0; i < MT; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = m0 + wm * WTM + i * 32 + (r >> 2) * 8 + g * 4 + (r & 3);
            if (m >= a.M) continue;
            const int64_t crow = a.c_rows ? (int64_t)a.c_rows[m] : (int64_t)m;
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                const int n = n0 + wn * WTN + j * 32 + li;
                if (n < a.N) {
                    float v = acc[i][j][r];
                    if (a.bias) v += a.bias[n];
                    if (a.relu) v = v > 0.f ? v : 0.f;
                    if (a.mask) v = post_elem<DT>(v, a.C, crow * a.ldc + n, m < a.n_acc, a.mask, crow * a.ldm + n);
                    store_elem<DT>(a.C, crow * a.ldc + n, v);
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// gemm_nt, wide tile.  The layer widths of the paper's models (128 .. 602) make these products
// "skinny": the reduction and the output width are both a few hundred, the row count is millions,
// so at bf16 the operand rows come from HBM faster than a small tile can turn them over.  This
// variant gives one workgroup 128 rows x the WHOLE output width (up to 256 columns: each operand
// row is read once), a wave 64 x 32*NTW, and moves 64-byte row slices through a double-buffered LDS
// ring with ONE barrier per slice: while slice s feeds the MFMAs, slice s+1 waits in registers and
// slice s+2 is in flight.  LDS rows are 64 bytes without padding; the 16-byte chunk c of row r sits
// at slot c ^ ((r >> 1) & 3), so that eight consecutive rows read with the same c touch eight
// different 16-byte bank groups.  Preconditions (checked by the launcher): 16-byte aligned operand
// rows and a reduction length that is a multiple of the slice; rows beyond M and columns beyond N
// are computed from clamped addresses and discarded.
// ------------------------------------------------------------------------------------------
// keeps the first n_valid elements of a 16-byte chunk, zeroes the rest (n_valid <= 0: all of it)
template <int DT>
__device__ __forceinline__ u32x4 mask_chunk(u32x4 r, int n_valid) {
    if (DT == GNN_F32) {
#pragma unroll
        for (int t = 0; t < 4; ++t) r[t] = n_valid > t ? r[t] : 0u;
    } else {
#pragma unroll
        for (int t = 0; t < 4; ++t) r[t] &= (n_valid > 2 * t ? 0xffffu : 0u) | (n_valid > 2 * t + 1 ? 0xffff0000u : 0u);
    }
    return r;
}

// KTAIL: the reduction length is not a multiple of the slice.  The last slice of every source is then cut: chunks
// that start at or beyond K are read from the start of their row instead (always addressable) and every chunk is
// masked to its valid elements when it is moved to LDS, so neither padding nor a neighbouring row reaches the MFMAs.
template <int DT, int NTW, bool KTAIL>
__global__ __launch_bounds__(256, 2) void gemm_nt_wide_kernel(GemmNT a) {
    constexpr int BM = 128, BN = 64 * NTW, MT = 2, NT = NTW, WTN = 32 * NTW;
    constexpr int ES = DTy<DT>::ES, EPV = DTy<DT>::EPV;
    constexpr int EPS = 64 / ES;                  // reduction elements per slice
    constexpr int A_CH = BM / 64, B_CH = BN / 64;  // 16-byte chunks per thread and slice
    constexpr int BUF = (BM + BN) * 16;            // words per ring buffer
    constexpr int CW = (256 / ES) < WTN ? (256 / ES) : WTN;  // columns of one staged output piece (<= 256 bytes)
    constexpr int CROW = CW * ES / 4 + 4;          // words per staged row (16 bytes of padding)
    constexpr int STAGE = 32 * CROW;               // words per wave
    constexpr int SMEM = 2 * BUF > 4 * STAGE ? 2 * BUF : 4 * STAGE;
    __shared__ __attribute__((aligned(16))) uint32_t smem[SMEM];
    // bias values and output rows of the tile, put here at the start: a load from global memory inside the epilogue
    // waits for the stores issued before it (see the line variant)
    __shared__ float s_bias[BN];
    __shared__ int32_t s_crow[BM];

    const int tiles_n = (a.N + BN - 1) / BN;
    const int m0 = (int)(blockIdx.x / tiles_n) * BM, n0 = (int)(blockIdx.x % tiles_n) * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, g = lane >> 5;
    const int ld_row = tid >> 2, ld_c = tid & 3;   // loader: row within a 64-row band, 16-byte chunk of the slice
    const int st_off = ld_row * 16 + ((ld_c ^ ((ld_row >> 1) & 3)) << 2);  // word offset of that chunk inside a band

    // per-thread operand rows as byte offsets (scalars, not arrays: everything here must stay in registers)
    auto a_row = [&](int c) -> int64_t {
        const int m = m0 + ld_row + 64 * c;
        const int64_t r = m < a.M ? (a.a_rows ? (int64_t)a.a_rows[m] : (int64_t)m) : (a.a_rows ? (int64_t)a.a_rows[0] : 0);
        return (r * a.lda + (KTAIL ? 0 : ld_c * EPV)) * ES;
    };
    auto b_row = [&](int c) -> int64_t {
        const int n = n0 + ld_row + 64 * c;
        return ((int64_t)(n < a.N ? n : 0) * a.ldb + (KTAIL ? 0 : ld_c * EPV)) * ES;
    };
    const int64_t ao0 = a_row(0), ao1 = a_row(1);
    const int64_t bo0 = b_row(0), bo1 = B_CH > 1 ? b_row(1) : 0, bo2 = B_CH > 2 ? b_row(2) : 0, bo3 = B_CH > 2 ? b_row(3) : 0;

    v16f acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int k_slices = KTAIL ? (a.K + EPS - 1) / EPS : a.K / EPS;
    const int n_steps = k_slices * ((a.n_src == 2 && m0 >= a.M1) ? 1 : a.n_src);   // a tile past M1 has one source only
    // rows of this thread's two chunks that lie at or past M1: their second-source data is zeroed on its way to LDS
    const bool z0 = m0 + ld_row >= a.M1, z1 = m0 + ld_row + 64 >= a.M1;
    // Everything that lives across steps is a plain variable filled and drained by macros (arrays handed to
    // helper functions ended up in scratch memory).  Two register sets (0, 1) hold the slices in flight from
    // global memory, two fragment sets (f0, f1) hold the operands of the two halves of a slice.
    u32x4 a0x0, a0x1, a1x0, a1x1;
    u32x4 b0x0, b0x1, b0x2, b0x3, b1x0, b1x1, b1x2, b1x3;
    u32x4 f0a0, f0a1, f0b0, f0b1, f0b2, f0b3, f1a0, f1a1, f1b0, f1b1, f1b2, f1b3;
    f1a0 = f1a1 = f1b0 = f1b1 = f1b2 = f1b3 = (u32x4){0u, 0u, 0u, 0u};
// a fetch beyond the last slice repeats the last one (a cache hit; what it brings is stashed but never multiplied)
#define GNN_FETCH(S, step_)                                                        \
    {                                                                              \
        const int st_ = (step_) < n_steps ? (step_) : n_steps - 1;                 \
        const int src_ = st_ >= k_slices ? 1 : 0;                                  \
        const int sl_ = st_ - src_ * k_slices;                                     \
        int64_t kb_ = (int64_t)sl_ * 64;                                           \
        if (KTAIL) kb_ = a.K - (sl_ * EPS + ld_c * EPV) > 0 ? kb_ + ld_c * 16 : 0; \
        const char* Ab_ = (const char*)(src_ ? a.A[1] : a.A[0]) + kb_;             \
        const char* Bb_ = (const char*)(src_ ? a.Bt[1] : a.Bt[0]) + kb_;           \
        a##S##x0 = *(const u32x4*)(Ab_ + ao0);                                     \
        a##S##x1 = *(const u32x4*)(Ab_ + ao1);                                     \
        b##S##x0 = *(const u32x4*)(Bb_ + bo0);                                     \
        if (B_CH > 1) b##S##x1 = *(const u32x4*)(Bb_ + bo1);                       \
        if (B_CH > 2) {                                                            \
            b##S##x2 = *(const u32x4*)(Bb_ + bo2);                                 \
            b##S##x3 = *(const u32x4*)(Bb_ + bo3);                                 \
        }                                                                          \
    }
#define GNN_STASH(buf_, S, step_)                                                  \
    {                                                                              \
        if (KTAIL) {                                                               \
            const int st_ = (step_) < n_steps ? (step_) : n_steps - 1;             \
            const int nv_ = a.K - ((st_ - (st_ >= k_slices ? k_slices : 0)) * EPS + ld_c * EPV); \
            a##S##x0 = mask_chunk<DT>(a##S##x0, nv_);                              \
            a##S##x1 = mask_chunk<DT>(a##S##x1, nv_);                              \
            b##S##x0 = mask_chunk<DT>(b##S##x0, nv_);                              \
            if (B_CH > 1) b##S##x1 = mask_chunk<DT>(b##S##x1, nv_);                \
            if (B_CH > 2) {                                                        \
                b##S##x2 = mask_chunk<DT>(b##S##x2, nv_);                          \
                b##S##x3 = mask_chunk<DT>(b##S##x3, nv_);                          \
            }                                                                      \
        }                                                                          \
        {                                                                          \
            const int sq_ = (step_) < n_steps ? (step_) : n_steps - 1;             \
            const bool s1_ = sq_ >= k_slices;                                      \
            a##S##x0 = (s1_ && z0) ? (u32x4){0u, 0u, 0u, 0u} : a##S##x0;           \
            a##S##x1 = (s1_ && z1) ? (u32x4){0u, 0u, 0u, 0u} : a##S##x1;           \
        }                                                                          \
        *(u32x4*)&(buf_)[st_off] = a##S##x0;                                       \
        *(u32x4*)&(buf_)[1024 + st_off] = a##S##x1;                                \
        *(u32x4*)&(buf_)[BM * 16 + st_off] = b##S##x0;                             \
        if (B_CH > 1) *(u32x4*)&(buf_)[BM * 16 + 1024 + st_off] = b##S##x1;        \
        if (B_CH > 2) {                                                            \
            *(u32x4*)&(buf_)[BM * 16 + 2048 + st_off] = b##S##x2;                  \
            *(u32x4*)&(buf_)[BM * 16 + 3072 + st_off] = b##S##x3;                  \
        }                                                                          \
    }
    // fragments: row (.. + li), chunk g*2+q of the slice
    const int sw = (li >> 1) & 3;
    const int fa_off = (wm * 64 + li) * 16, fb_off = BM * 16 + (wn * WTN + li) * 16;
    const int slot0 = ((g * 2) ^ sw) << 2, slot1 = ((g * 2 + 1) ^ sw) << 2;
#define GNN_READ(F, buf_, slot_)                                                   \
    {                                                                              \
        F##a0 = *(const u32x4*)&(buf_)[fa_off + (slot_)];                          \
        F##a1 = *(const u32x4*)&(buf_)[fa_off + 512 + (slot_)];                    \
        F##b0 = *(const u32x4*)&(buf_)[fb_off + (slot_)];                          \
        if (NT > 1) F##b1 = *(const u32x4*)&(buf_)[fb_off + 512 + (slot_)];        \
        if (NT > 2) {                                                              \
            F##b2 = *(const u32x4*)&(buf_)[fb_off + 1024 + (slot_)];               \
            F##b3 = *(const u32x4*)&(buf_)[fb_off + 1536 + (slot_)];               \
        }                                                                          \
    }
    auto mma = [&](v16f& c, const u32x4& x, const u32x4& y) {
        if (DT == GNN_F32) {
#pragma unroll
            for (int t = 0; t < 4; ++t) c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(x[t]), __uint_as_float(y[t]), c, 0, 0, 0);
        } else {
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, x), __builtin_bit_cast(v8bf, y), c, 0, 0, 0);
        }
    };
#define GNN_MMA(F)                                                                 \
    {                                                                              \
        mma(acc[0][0], F##a0, F##b0);                                              \
        mma(acc[1][0], F##a1, F##b0);                                              \
        if (NT > 1) {                                                              \
            mma(acc[0][NT > 1 ? 1 : 0], F##a0, F##b1);                             \
            mma(acc[1][NT > 1 ? 1 : 0], F##a1, F##b1);                             \
        }                                                                          \
        if (NT > 2) {                                                              \
            mma(acc[0][NT > 2 ? 2 : 0], F##a0, F##b2);                             \
            mma(acc[1][NT > 2 ? 2 : 0], F##a1, F##b2);                             \
            mma(acc[0][NT > 2 ? 3 : 0], F##a0, F##b3);                             \
            mma(acc[1][NT > 2 ? 3 : 0], F##a1, F##b3);                             \
        }                                                                          \
    }
// One step on slice s_ (in ring buffer bufc_).  The second half of the previous slice is still waiting in f1: its
// MFMAs run while the first half of this slice comes from LDS, and the MFMAs of the first half run while the second
// half comes - LDS latency is hidden inside one wave.  Nothing here is conditional: with branches around the loads
// or the LDS writes the compiler's wait-counter tracking loses the order of the outstanding loads.
#define GNN_STEP(s_, bufc_, bufn_, SF, SS)                                         \
    {                                                                              \
        GNN_READ(f0, bufc_, slot0)                                                 \
        GNN_FETCH(SF, (s_) + 2)                                                    \
        __builtin_amdgcn_sched_barrier(0);                                         \
        GNN_MMA(f1)                                                                \
        __builtin_amdgcn_sched_barrier(0);                                         \
        GNN_READ(f1, bufc_, slot1)                                                 \
        __builtin_amdgcn_sched_barrier(0);                                         \
        GNN_MMA(f0)                                                                \
        __builtin_amdgcn_sched_barrier(0);                                         \
        GNN_STASH(bufn_, SS, (s_) + 1)                                             \
        __syncthreads();                                                           \
    }
    uint32_t* buf0 = smem;
    uint32_t* buf1 = smem + BUF;
    // invariant at the top of step s: ring buffer s%2 holds slice s (visible to all waves), register set (s+1)%2 holds
    // slice s+1 (possibly still in flight), register set s%2 is free, f1 holds the second half of slice s-1 (zeros at first)
    GNN_FETCH(0, 0)
    GNN_FETCH(1, 1)
    {
        const int n = n0 + (tid & (BN - 1)), m = m0 + (tid & (BM - 1));
        s_bias[tid & (BN - 1)] = (a.bias && n < a.N) ? a.bias[n] : 0.f;
        s_crow[tid & (BM - 1)] = m < a.M ? (a.c_rows ? a.c_rows[m] : m) : -1;   // -1: a row past M, never stored
    }
    GNN_STASH(buf0, 0, 0)
    __syncthreads();
    const int n_pairs = n_steps >> 1;
    for (int pr = 0; pr < n_pairs; ++pr) {
        const int step = pr << 1;
        GNN_STEP(step, buf0, buf1, 0, 1)
        GNN_STEP(step + 1, buf1, buf0, 1, 0)
    }
    if (n_steps & 1) GNN_STEP(n_steps - 1, buf0, buf1, 0, 1)
    GNN_MMA(f1)
#undef GNN_FETCH
#undef GNN_STASH
#undef GNN_READ
#undef GNN_MMA
#undef GNN_STEP

    // Epilogue.  acc[i][j][r] is C[row (r/4)*8 + g*4 + r%4][column li] of its 32x32 block: a piece of 32 rows x CW
    // columns is laid out row-major in the wave's part of LDS (bias, ReLU and rounding applied) and written with
    // 16-byte stores, up to 256 contiguous bytes per row.
    uint32_t* stg = smem + wave * STAGE;
    constexpr int JP = CW / 32;            // 32-column blocks per piece
    constexpr int CPR = CW * ES / 16;      // 16-byte chunks per staged row
    constexpr int RPP = 64 / CPR;          // rows written per pass of the wave
#pragma unroll
    for (int i = 0; i < MT; ++i) {
#pragma unroll
        for (int p = 0; p < NT / JP; ++p) {
#pragma unroll
            for (int jj = 0; jj < JP; ++jj) {
                const int j = p * JP + jj;
                const float bv = s_bias[wn * WTN + j * 32 + li];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = (r >> 2) * 8 + g * 4 + (r & 3);
                    float v = acc[i][j][r] + bv;
                    if (a.relu) v = v > 0.f ? v : 0.f;
                    if (DT == GNN_F32) stg[row * CROW + jj * 32 + li] = __float_as_uint(v);
                    else ((uint16_t*)stg)[row * (CROW * 2) + jj * 32 + li] = f32_to_bf16(v);
                }
            }
            __syncthreads();
#pragma unroll
            for (int pass = 0; pass < 32 / RPP; ++pass) {
                const int row = pass * RPP + lane / CPR, ch = lane % CPR;
                const int m = m0 + wm * 64 + i * 32 + row;
                const int n = n0 + wn * WTN + p * CW + ch * EPV;
                const int64_t crow = s_crow[wm * 64 + i * 32 + row];
                if (crow >= 0 && n < a.N) {
                    uint4 v = *(const uint4*)&stg[row * CROW + ch * 4];
                    char* dst = (char*)a.C + (crow * a.ldc + n) * ES;
                    if (n + EPV <= a.N && a.c_vec && (!a.mask || a.m_vec)) {
                        if (a.mask) v = post_vec<DT>(v, a.C, crow * a.ldc + n, m < a.n_acc, a.mask, crow * a.ldm + n);
                        *(uint4*)dst = v;
                    } else {
                        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
                        if (DT == GNN_F32) {
                            for (int e = 0; e < 4 && n + e < a.N; ++e) {
                                float o = __uint_as_float(w[e]);
                                if (a.mask) o = post_elem<DT>(o, a.C, crow * a.ldc + n + e, m < a.n_acc, a.mask, crow * a.ldm + n + e);
                                ((float*)dst)[e] = o;
                            }
                        } else {
                            for (int e = 0; e < 8 && n + e < a.N; ++e) {
                                uint16_t o = (uint16_t)(w[e >> 1] >> ((e & 1) * 16));
                                if (a.mask) o = f32_to_bf16(post_elem<DT>(bf16_to_f32(o), a.C, crow * a.ldc + n + e, m < a.n_acc, a.mask, crow * a.ldm + n + e));
                                ((uint16_t*)dst)[e] = o;
                            }
                        }
                    }
                }
            }
            __syncthreads();
        }
    }
}

// ------------------------------------------------------------------------------------------
// gemm_nt, line tile.  Same tile as the wide variant (128 rows x the whole output width, a wave
// 64 x 32*NTW), two things done differently.
// (1) The reduction moves in slices of 128 bytes - one whole cache line of every operand row.  With
// 64-byte slices every line is asked for twice, one step apart, and by then it has left the CU's
// vector cache: the L2 sees two requests per line.  A slice of this size leaves room for ONE copy in
// LDS (48 KB at 256 columns, two workgroups per CU), so a step has two barriers: slice s feeds the
// MFMAs while slice s+1 is in flight into registers; barrier; the registers go to LDS; barrier.  The
// other workgroup of the CU computes meanwhile, and the last quarter of a slice is multiplied while
// the first quarter of the next one comes from LDS.  LDS rows are 128 bytes without padding; the
// 16-byte chunk c of row r sits at slot c ^ ((r >> 1) & 7): sixteen consecutive rows read with the
// same c touch all 64 banks once.
// (2) The epilogue never waits for memory.  A short reduction (2 .. 8 steps at the paper's widths)
// leaves the epilogue a third of a tile's time, and most of that was waiting: loads and stores share
// one counter on this chip, so any load inside the epilogue (a bias value, an output row index, and
// the wait the compiler puts where a branch around such a load rejoins) stalls until the stores
// before it have landed.  Here the bias and the output rows are put in LDS when the tile starts, LDS
// reads are issued in batches ahead of their use, the activation mask of a fused input gradient is
// loaded for all rows of a pass before the first store of that pass, and the MFMAs run with the
// operands exchanged so that a lane holds four CONSECUTIVE columns of one row (8- or 16-byte LDS
// writes instead of 2-byte ones).
// Preconditions (checked by the launcher, which sends everything else to the wide variant): 16-byte
// aligned operand, output and mask rows, a reduction length that is a multiple of the slice, an
// output width that is a multiple of the tile width.
// ------------------------------------------------------------------------------------------
template <int DT, int NTW>
__global__ __launch_bounds__(256, NTW == 4 ? 2 : 3) void gemm_nt_line_kernel(GemmNT a) {
    constexpr int BM = 128, BN = 64 * NTW, MT = 2, NT = NTW, WTN = 32 * NTW;
    constexpr int ES = DTy<DT>::ES, EPV = DTy<DT>::EPV;
    constexpr int EPS = 128 / ES;                  // reduction elements per slice
    constexpr int B_CH = BN / 32;                  // 16-byte chunks of the second operand per thread and slice (first: 4)
    constexpr int BUF = (BM + BN) * 32;            // words of the slice buffer
    constexpr int CW = (256 / ES) < WTN ? (256 / ES) : WTN;  // columns of one staged output piece (<= 256 bytes)
    constexpr int CROW = CW * ES / 4 + 4;          // words per staged row (16 bytes of padding)
    constexpr int STAGE = 32 * CROW;               // words per wave
    constexpr int SMEM = BUF > 4 * STAGE ? BUF : 4 * STAGE;
    __shared__ __attribute__((aligned(16))) uint32_t smem[SMEM];
    // The tile's bias values and output rows wait in LDS: read from global memory inside the epilogue, each of them
    // would make the wave wait for EVERY vector-memory operation it has in flight - that is, for the stores of the rows
    // before - because one counter covers loads and stores alike.
    __shared__ float s_bias[BN];
    __shared__ int32_t s_crow[BM];

    const int tiles_n = a.N / BN;
        const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, g = lane >> 5;
    const int ld_row = tid >> 3, ld_c = tid & 7;   // loader: row within a 32-row band, 16-byte chunk of the slice
    const int st_off = ld_row * 32 + ((ld_c ^ ((ld_row >> 1) & 7)) << 2);  // word offset of that chunk inside a band
    const int k_slices = a.K / EPS;
    // the tile's rows of the second operand are all in range (N is a multiple of BN): band c lies c * 32 rows further
    const int64_t b_band = 32 * a.ldb * ES;

    const int m0 = (int)(blockIdx.x / tiles_n) * BM, n0 = (int)(blockIdx.x % tiles_n) * BN;
    // operand row of the loader's band c (rows past M read an addressable row; their results are never stored)
    auto a_row = [&](int c) -> int64_t {
        const int m = m0 + ld_row + 32 * c;
        const int64_t r = m < a.M ? (a.a_rows ? (int64_t)a.a_rows[m] : (int64_t)m) : (a.a_rows ? (int64_t)a.a_rows[0] : 0);
        return (r * a.lda + ld_c * EPV) * ES;
    };
    const int64_t ao0 = a_row(0), ao1 = a_row(1), ao2 = a_row(2), ao3 = a_row(3);
    const int64_t bo0 = ((int64_t)(n0 + ld_row) * a.ldb + ld_c * EPV) * ES;
    const int n_steps = k_slices * ((a.n_src == 2 && m0 >= a.M1) ? 1 : a.n_src);   // a tile past M1 has one source only
    // rows of this thread's chunks that lie at or past M1: their second-source data is zeroed on its way to LDS
    const bool z0 = m0 + ld_row >= a.M1, z1 = m0 + ld_row + 32 >= a.M1, z2 = m0 + ld_row + 64 >= a.M1, z3 = m0 + ld_row + 96 >= a.M1;

    v16f acc[MT][NT];
    // plain variables filled and drained by macros, as in the wide variant: one register set for the slice in flight,
    // two fragment sets (f0, f1) for alternating quarters of a slice
    u32x4 ax0, ax1, ax2, ax3;
    u32x4 bx0, bx1, bx2, bx3, bx4, bx5, bx6, bx7;
    u32x4 f0a0, f0a1, f0b0, f0b1, f0b2, f0b3, f1a0, f1a1, f1b0, f1b1, f1b2, f1b3;
    f0b1 = f0b2 = f0b3 = (u32x4){0u, 0u, 0u, 0u};
    f1a0 = f1a1 = f1b0 = f1b1 = f1b2 = f1b3 = (u32x4){0u, 0u, 0u, 0u};
    bx4 = bx5 = bx6 = bx7 = (u32x4){0u, 0u, 0u, 0u};
// a fetch beyond the last slice repeats the last one (a cache hit; what it brings is stashed but never multiplied)
#define GNN_FETCH(step_)                                                           \
    {                                                                              \
        const int st_ = (step_) < n_steps ? (step_) : n_steps - 1;                 \
        const int src_ = st_ >= k_slices ? 1 : 0;                                  \
        const int64_t kb_ = (int64_t)(st_ - src_ * k_slices) * 128;                \
        const char* Ab_ = (const char*)(src_ ? a.A[1] : a.A[0]) + kb_;             \
        const char* Bb_ = (const char*)(src_ ? a.Bt[1] : a.Bt[0]) + kb_ + bo0;     \
        ax0 = *(const u32x4*)(Ab_ + ao0);                                          \
        ax1 = *(const u32x4*)(Ab_ + ao1);                                          \
        ax2 = *(const u32x4*)(Ab_ + ao2);                                          \
        ax3 = *(const u32x4*)(Ab_ + ao3);                                          \
        bx0 = *(const u32x4*)(Bb_);                                                \
        bx1 = *(const u32x4*)(Bb_ + b_band);                                       \
        bx2 = *(const u32x4*)(Bb_ + 2 * b_band);                                   \
        bx3 = *(const u32x4*)(Bb_ + 3 * b_band);                                   \
        if (B_CH > 4) {                                                            \
            bx4 = *(const u32x4*)(Bb_ + 4 * b_band);                               \
            bx5 = *(const u32x4*)(Bb_ + 5 * b_band);                               \
            bx6 = *(const u32x4*)(Bb_ + 6 * b_band);                               \
            bx7 = *(const u32x4*)(Bb_ + 7 * b_band);                               \
        }                                                                          \
    }
#define GNN_STASH(step_)                                                           \
    {                                                                              \
        const int sq_ = (step_) < n_steps ? (step_) : n_steps - 1;                 \
        const bool s1_ = sq_ >= k_slices;                                          \
        *(u32x4*)&smem[st_off] = (s1_ && z0) ? (u32x4){0u, 0u, 0u, 0u} : ax0;      \
        *(u32x4*)&smem[1024 + st_off] = (s1_ && z1) ? (u32x4){0u, 0u, 0u, 0u} : ax1; \
        *(u32x4*)&smem[2048 + st_off] = (s1_ && z2) ? (u32x4){0u, 0u, 0u, 0u} : ax2; \
        *(u32x4*)&smem[3072 + st_off] = (s1_ && z3) ? (u32x4){0u, 0u, 0u, 0u} : ax3; \
        *(u32x4*)&smem[BM * 32 + st_off] = bx0;                                    \
        *(u32x4*)&smem[BM * 32 + 1024 + st_off] = bx1;                             \
        *(u32x4*)&smem[BM * 32 + 2048 + st_off] = bx2;                             \
        *(u32x4*)&smem[BM * 32 + 3072 + st_off] = bx3;                             \
        if (B_CH > 4) {                                                            \
            *(u32x4*)&smem[BM * 32 + 4096 + st_off] = bx4;                         \
            *(u32x4*)&smem[BM * 32 + 5120 + st_off] = bx5;                         \
            *(u32x4*)&smem[BM * 32 + 6144 + st_off] = bx6;                         \
            *(u32x4*)&smem[BM * 32 + 7168 + st_off] = bx7;                         \
        }                                                                          \
    }
    // fragments: row (.. + li), chunk g*4 + q of the slice for quarter q (the same permutation of the reduction index
    // in both operands, which leaves the product unchanged)
    const int sw = (li >> 1) & 7;
    const int fa_off = (wm * 64 + li) * 32, fb_off = BM * 32 + (wn * WTN + li) * 32;
#define GNN_READ(F, q_)                                                            \
    {                                                                              \
        const int slot_ = ((g * 4 + (q_)) ^ sw) << 2;                              \
        F##a0 = *(const u32x4*)&smem[fa_off + slot_];                              \
        F##a1 = *(const u32x4*)&smem[fa_off + 1024 + slot_];                       \
        F##b0 = *(const u32x4*)&smem[fb_off + slot_];                              \
        if (NT > 1) F##b1 = *(const u32x4*)&smem[fb_off + 1024 + slot_];           \
        if (NT > 2) {                                                              \
            F##b2 = *(const u32x4*)&smem[fb_off + 2048 + slot_];                   \
            F##b3 = *(const u32x4*)&smem[fb_off + 3072 + slot_];                   \
        }                                                                          \
    }
    auto mma = [&](v16f& c, const u32x4& x, const u32x4& y) {
        if (DT == GNN_F32) {
#pragma unroll
            for (int t = 0; t < 4; ++t) c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(x[t]), __uint_as_float(y[t]), c, 0, 0, 0);
        } else {
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, x), __builtin_bit_cast(v8bf, y), c, 0, 0, 0);
        }
    };
#define GNN_MMA(F)                                                                 \
    {                                                                              \
        mma(acc[0][0], F##b0, F##a0);                                              \
        mma(acc[1][0], F##b0, F##a1);                                              \
        if (NT > 1) {                                                              \
            mma(acc[0][NT > 1 ? 1 : 0], F##b1, F##a0);                             \
            mma(acc[1][NT > 1 ? 1 : 0], F##b1, F##a1);                             \
        }                                                                          \
        if (NT > 2) {                                                              \
            mma(acc[0][NT > 2 ? 2 : 0], F##b2, F##a0);                             \
            mma(acc[1][NT > 2 ? 2 : 0], F##b2, F##a1);                             \
            mma(acc[0][NT > 2 ? 3 : 0], F##b3, F##a0);                             \
            mma(acc[1][NT > 2 ? 3 : 0], F##b3, F##a1);                             \
        }                                                                          \
    }
// the four quarters of the slice in LDS: the first fragments (f0) are on their way; f1 still holds the last quarter
// of the slice before
#define GNN_QUARTERS                                                               \
    {                                                                              \
        __builtin_amdgcn_sched_barrier(0);                                         \
        GNN_MMA(f1)                                                                \
        __builtin_amdgcn_sched_barrier(0);                                         \
        GNN_READ(f1, 1)                                                            \
        __builtin_amdgcn_sched_barrier(0);                                         \
        GNN_MMA(f0)                                                                \
        __builtin_amdgcn_sched_barrier(0);                                         \
        GNN_READ(f0, 2)                                                            \
        __builtin_amdgcn_sched_barrier(0);                                         \
        GNN_MMA(f1)                                                                \
        __builtin_amdgcn_sched_barrier(0);                                         \
        GNN_READ(f1, 3)                                                            \
        __builtin_amdgcn_sched_barrier(0);                                         \
        GNN_MMA(f0)                                                                \
        __builtin_amdgcn_sched_barrier(0);                                         \
    }
    // invariant at the top of step s: LDS holds slice s (visible to all waves), the register set is free, f1 holds the
    // last quarter of slice s-1 (zeros at first).  Nothing in a step is conditional (see the wide variant).
    GNN_FETCH(0)
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    f1a0 = f1a1 = f1b0 = f1b1 = f1b2 = f1b3 = (u32x4){0u, 0u, 0u, 0u};
    s_bias[tid & (BN - 1)] = a.bias ? a.bias[n0 + (tid & (BN - 1))] : 0.f;   // arrives with the slice the stash waits for
    {
        const int m = m0 + (tid & (BM - 1));
        s_crow[tid & (BM - 1)] = m < a.M ? (a.c_rows ? a.c_rows[m] : m) : -1;   // -1: a row past M, never stored
    }
    GNN_STASH(0)
    __syncthreads();
    for (int s = 0; s < n_steps; ++s) {
        GNN_READ(f0, 0)
        GNN_FETCH(s + 1)
        GNN_QUARTERS
        __syncthreads();          // every wave has taken its fragments of slice s
        GNN_STASH(s + 1)
        __syncthreads();
    }
    GNN_MMA(f1)

    // Epilogue.  The MFMAs ran with the operands exchanged (the weights' rows as the first operand): acc[i][j][r] is
    // C[row li][column (r/4)*8 + g*4 + r%4] of its 32x32 block, four consecutive columns per lane and r/4.  A piece of
    // 32 rows x CW columns is laid out row-major in the wave's part of LDS with 8- or 16-byte writes (bias, ReLU and
    // rounding applied) and written to memory with 16-byte stores, up to 256 contiguous bytes per row.
    uint32_t* stg = smem + wave * STAGE;
    constexpr int JP = CW / 32;            // 32-column blocks per piece
    constexpr int CPR = CW * ES / 16;      // 16-byte chunks per staged row
    constexpr int RPP = 64 / CPR;          // rows written per pass of the wave
    // what the epilogue needs from LDS is asked for in batches ahead of its use: a read issued right before its
    // use costs one LDS round trip each time, and sixteen of those in a row were most of the epilogue
    float4 bvs[NT][4];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) bvs[j][q] = *(const float4*)&s_bias[wn * WTN + j * 32 + q * 8 + g * 4];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
#pragma unroll
        for (int p = 0; p < NT / JP; ++p) {
#pragma unroll
            for (int jj = 0; jj < JP; ++jj) {
                const int j = p * JP + jj;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int c = q * 8 + g * 4;     // first of this lane's four consecutive columns of the block
                    const float4 bv = bvs[j][q];
                    float v0 = acc[i][j][q * 4 + 0] + bv.x, v1 = acc[i][j][q * 4 + 1] + bv.y;
                    float v2 = acc[i][j][q * 4 + 2] + bv.z, v3 = acc[i][j][q * 4 + 3] + bv.w;
                    if (a.relu) {
                        v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f);
                    }
                    if (DT == GNN_F32) {
                        *(uint4*)&stg[li * CROW + jj * 32 + c] = make_uint4(__float_as_uint(v0), __float_as_uint(v1), __float_as_uint(v2), __float_as_uint(v3));
                    } else {
                        *(uint2*)&stg[li * CROW + jj * 16 + (c >> 1)] = make_uint2(pack_bf16(v0, v1), pack_bf16(v2, v3));
                    }
                }
            }
            __syncthreads();
            constexpr int NP = 32 / RPP;   // passes of the wave over the piece
            const int n = n0 + wn * WTN + p * CW + (lane % CPR) * EPV;
            int32_t crs[NP];
            uint4 vs[NP];
#pragma unroll
            for (int pass = 0; pass < NP; ++pass) {
                const int row = pass * RPP + lane / CPR;
                crs[pass] = s_crow[wm * 64 + i * 32 + row];
                vs[pass] = *(const uint4*)&stg[row * CROW + (lane % CPR) * 4];
            }
            // 16-byte stores only: the launcher sends other layouts to the wide variant
            if (a.mask) {
                // the activation mask (and, for the rows that accumulate, what C holds) of all passes first, then the
                // stores: a load between two stores would wait for the store before it
                uint4 hs[NP], os[NP];
#pragma unroll
                for (int pass = 0; pass < NP; ++pass) {
                    const int64_t crow = crs[pass] >= 0 ? crs[pass] : 0;      // a row past M reads an addressable row
                    const int m = m0 + wm * 64 + i * 32 + pass * RPP + lane / CPR;
                    hs[pass] = *(const uint4*)((const char*)a.mask + (crow * a.ldm + n) * ES);
                    os[pass] = make_uint4(0u, 0u, 0u, 0u);
                    if (m < a.n_acc) os[pass] = *(const uint4*)((const char*)a.C + (crow * a.ldc + n) * ES);
                }
#pragma unroll
                for (int pass = 0; pass < NP; ++pass) {
                    const int m = m0 + wm * 64 + i * 32 + pass * RPP + lane / CPR;
                    vs[pass] = post_apply<DT>(vs[pass], os[pass], m < a.n_acc, hs[pass]);
                }
            }
#pragma unroll
            for (int pass = 0; pass < NP; ++pass) {
                const int64_t crow = crs[pass];
                if (crow >= 0) *(uint4*)((char*)a.C + (crow * a.ldc + n) * ES) = vs[pass];
            }
            __syncthreads();
        }
    }
#undef GNN_FETCH
#undef GNN_STASH
#undef GNN_READ
#undef GNN_MMA
#undef GNN_QUARTERS
}

template <int DT>
static int32_t launch_gemm_nt(const GemmNT& a, hipStream_t stream) {
    if (a.M <= 0 || a.N <= 0) return GNN_OK;
    const int64_t tiles_m = ((int64_t)a.M + 127) / 128;
    const bool vec = a.a_vec && a.b_vec;  // both operands aligned: the branch-free loader
    if (vec && a.N > 32 && a.K > 0) {
        // wide tile: the tile width that pads the output width least (256 on a tie)
        const int64_t p256 = ((int64_t)a.N + 255) / 256 * 256, p128 = ((int64_t)a.N + 127) / 128 * 128, p64 = ((int64_t)a.N + 63) / 64 * 64;
        int ntw = (p256 <= p128 && p256 <= p64) ? 4 : (p128 <= p64 ? 2 : 1);
        // a reduction of one or two slices (an input gradient from 32 or 41 class scores) is all prologue and epilogue:
        // narrow tiles keep more workgroups on a CU to hide those latencies, and re-reading the short rows costs little
        if ((int64_t)a.K * a.n_src * DTy<DT>::ES <= 128) ntw = 1;
        // whole cache lines per step where the shapes allow it (see gemm_nt_line_kernel)
#ifndef GNN_NT_LINE
#define GNN_NT_LINE 1
#endif
// fp32 products are bound by the fp32 MFMA rate, not by requests or the epilogue: the line tile changed none of
// their durations (configs[1] and [2]), so they stay on the wide variant
#ifndef GNN_NT_LINE_F32
#define GNN_NT_LINE_F32 0
#endif
        if constexpr (GNN_NT_LINE && (DT == GNN_BF16 || GNN_NT_LINE_F32))
        if ((int64_t)a.K * DTy<DT>::ES % 128 == 0 && ntw > 1 && a.N % (64 * ntw) == 0 && a.c_vec && (!a.mask || a.m_vec)) {
            const unsigned lgrid = (unsigned)(tiles_m * (a.N / (64 * ntw)));
            if (ntw == 4) gemm_nt_line_kernel<DT, 4><<<lgrid, 256, 0, stream>>>(a);
            else gemm_nt_line_kernel<DT, 2><<<lgrid, 256, 0, stream>>>(a);
            GNN_LAUNCH_CHECK("gemm_nt_line_kernel");
            return GNN_OK;
        }
        const unsigned grid = (unsigned)(tiles_m * (ntw == 4 ? p256 / 256 : (ntw == 2 ? p128 / 128 : p64 / 64)));
        const bool ktail = a.K % (64 / DTy<DT>::ES) != 0;
#define GNN_WIDE(NTW_)                                                                                  \
    {                                                                                                   \
        if (ktail) gemm_nt_wide_kernel<DT, NTW_, true><<<grid, 256, 0, stream>>>(a);                    \
        else gemm_nt_wide_kernel<DT, NTW_, false><<<grid, 256, 0, stream>>>(a);                         \
    }
        if (ntw == 4) GNN_WIDE(4)
        else if (ntw == 2) GNN_WIDE(2)
        else GNN_WIDE(1)
#undef GNN_WIDE
        GNN_LAUNCH_CHECK("gemm_nt_wide_kernel");
        return GNN_OK;
    }
    if (a.N > 64) {
        const unsigned grid = (unsigned)((tiles_m * ((a.N + 127) / 128) + 7) / 8 * 8);
        if (vec) gemm_nt_kernel<DT, 128, 2, 2, true><<<grid, 256, 0, stream>>>(a);
        else gemm_nt_kernel<DT, 128, 2, 2, false><<<grid, 256, 0, stream>>>(a);
    } else if (a.N > 32) {
        const unsigned grid = (unsigned)((tiles_m * ((a.N + 63) / 64) + 7) / 8 * 8);
        if (vec) gemm_nt_kernel<DT, 64, 2, 2, true><<<grid, 256, 0, stream>>>(a);
        else gemm_nt_kernel<DT, 64, 2, 2, false><<<grid, 256, 0, stream>>>(a);
    } else {
        const unsigned grid = (unsigned)((tiles_m + 7) / 8 * 8);
        if (vec) gemm_nt_kernel<DT, 32, 4, 1, true><<<grid, 256, 0, stream>>>(a);
        else gemm_nt_kernel<DT, 32, 4, 1, false><<<grid, 256, 0, stream>>>(a);
    }
    GNN_LAUNCH_CHECK("gemm_nt_kernel");
    return GNN_OK;
}

// ------------------------------------------------------------------------------------------
// gemm_tn : P[split][src*K + k][n] = sum_{m in split} A_src[row(m)][k] * D[m][n]
// ------------------------------------------------------------------------------------------
// Output tiles of the weight-gradient product are 128 x 256 instead of 128 x 128 where the width allows it (bf16: the
// fp32 product is bound by its MFMAs): the kernel runs at the rate its operand slabs come from L2 - 9.3 TB/s at every
// shape measured - and a slab of A is then fetched by one workgroup per split instead of two.
static inline bool tn_wide_columns(int dtype, int32_t N) { return dtype == GNN_BF16 && N >= 256 && N % 256 == 0; }

struct GemmTN {
    const void* A[2];
    int32_t n_src;
    int64_t lda;
    int32_t a_vec;
    const int32_t* a_rows;  // nullable
    const void* D;          // [M, ldd], rows compact
    int64_t ldd;
    int32_t d_vec;
    int32_t M, N, K;
    int32_t rows_per_split; // multiple of 32
    int32_t n_splits;
    float* P;               // [splits][n_src*K][N]
    float* Pb;              // nullable: [splits][N] column sums of D over each split (the bias gradient's partial sums)
};

template <int DT, int BN, bool VEC>
__global__ __launch_bounds__(256, BN == 256 ? 2 : 3) void gemm_tn_kernel(GemmTN a) {
    constexpr int BKO = 128, BMR = 32;
    constexpr int EPV = DTy<DT>::EPV;
    constexpr int WKO = BN >= 128 ? 2 : 4, WNN = 4 / WKO;      // waves along k-out and n
    constexpr int WTK = BKO / WKO, WTN = BN / WNN, MT = WTK / 32, NT = WTN / 32;
    constexpr int A_VPR = BKO / EPV;                 // 16-byte vectors per tile row
    constexpr int D_VPR = BN / EPV;
    constexpr int A_CH = BMR * A_VPR / 256;          // vectors per thread
    constexpr int D_CH = (BMR * D_VPR + 255) / 256;
    // LDS row strides in words: 32 bytes of padding put the four rows that one 16-lane group of a transpose read
    // touches into different bank groups
    constexpr int A_LDW = BKO * DTy<DT>::ES / 4 + 8, D_LDW = BN * DTy<DT>::ES / 4 + 8;
    __shared__ uint32_t sA[BMR * A_LDW];
    __shared__ uint32_t sD[BMR * D_LDW];
    __shared__ float s_bs[BMR * D_VPR * EPV];   // column sums of D, per tile row, before they are added up

    const int ko_tiles = (a.K + BKO - 1) / BKO;
    const int n_tiles = (a.N + BN - 1) / BN;
    // all tiles of one row split are consecutive logical ids, hence on one XCD: its L2 serves the re-reads
    const int tiles = a.n_src * ko_tiles * n_tiles;
    const int64_t total = (int64_t)tiles * a.n_splits;
    const int64_t logical = xcd_remap(blockIdx.x, total);
    if (logical >= total) return;
    const int t = (int)(logical % tiles);
    const int split = (int)(logical / tiles);
    const int tn = t % n_tiles, tk = (t / n_tiles) % ko_tiles, src = t / (n_tiles * ko_tiles);
    const int ko0 = tk * BKO, n0 = tn * BN;
    const int64_t m_begin = (int64_t)split * a.rows_per_split;
    const int64_t m_end = m_begin + a.rows_per_split < a.M ? m_begin + a.rows_per_split : a.M;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wk = wave / WNN, wn = wave % WNN;
    const int li = lane & 31, g = lane >> 5;
    const void* Ab = a.A[src];

    v16f acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // the workgroups of the first k-tile of the first source also add up the columns of D (each thread keeps the sums
    // of the chunk positions it loads; tile rows are added in order afterwards)
    const bool do_bias = a.Pb != nullptr && src == 0 && tk == 0;
    float bs[D_CH][EPV];
#pragma unroll
    for (int c = 0; c < D_CH; ++c)
#pragma unroll
        for (int e = 0; e < EPV; ++e) bs[c][e] = 0.f;
    uint4 ra[A_CH], rd[D_CH];
    auto fetch = [&](int64_t mb) {
#pragma unroll
        for (int c = 0; c < A_CH; ++c) {
            const int v = tid + 256 * c;
            const int row = v / A_VPR, kc = v % A_VPR;
            const int64_t m = mb + row;
            const int ke = ko0 + kc * EPV;
            int64_t r = 0;
            if (m < m_end) r = a.a_rows ? (int64_t)a.a_rows[m] : m;
            if (VEC) ra[c] = load_raw<DT>(Ab, r * a.lda + ke, m < m_end && ke < a.K);
            else ra[c] = load16<DT>(Ab, r * a.lda + ke, m < m_end ? a.K - ke : 0, a.a_vec != 0);
        }
#pragma unroll
        for (int c = 0; c < D_CH; ++c) {
            const int v = tid + 256 * c;
            const int row = v / D_VPR, nc = v % D_VPR;
            const int64_t m = mb + row;
            const int ne = n0 + nc * EPV;
            const bool ok = row < BMR && m < m_end;
            if (VEC) rd[c] = load_raw<DT>(a.D, m * a.ldd + ne, ok && ne < a.N);
            else rd[c] = load16<DT>(a.D, (ok ? m : 0) * a.ldd + ne, ok ? a.N - ne : 0, a.d_vec != 0);
        }
    };
    // `mb` is the first row of the tile being moved to LDS; out-of-range parts are zeroed here (VEC path)
    auto stash = [&](int64_t mb) {
        const bool edge = mb + BMR > m_end || ko0 + BKO > a.K || n0 + BN > a.N;  // uniform
#pragma unroll
        for (int c = 0; c < A_CH; ++c) {
            const int v = tid + 256 * c;
            if (VEC && edge) ra[c] = fix_chunk<DT>(ra[c], mb + v / A_VPR < m_end ? a.K - (ko0 + (v % A_VPR) * EPV) : 0);
            *(uint4*)&sA[(v / A_VPR) * A_LDW + (v % A_VPR) * 4] = ra[c];
        }
#pragma unroll
        for (int c = 0; c < D_CH; ++c) {
            const int v = tid + 256 * c;
            if (VEC && edge) rd[c] = fix_chunk<DT>(rd[c], mb + v / D_VPR < m_end ? a.N - (n0 + (v % D_VPR) * EPV) : 0);
            if (v / D_VPR < BMR) *(uint4*)&sD[(v / D_VPR) * D_LDW + (v % D_VPR) * 4] = rd[c];
            if (do_bias && v / D_VPR < BMR) {
                const uint32_t w[4] = {rd[c].x, rd[c].y, rd[c].z, rd[c].w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (DT == GNN_F32) {
                        bs[c][q] += __uint_as_float(w[q]);
                    } else {
                        bs[c][2 * q] += bf16lo(w[q]);
                        bs[c][2 * q + 1] += bf16hi(w[q]);
                    }
                }
            }
        }
    };

    if (m_begin < m_end) {
        fetch(m_begin);
        stash(m_begin);
    }
    __syncthreads();
    for (int64_t mb = m_begin; mb < m_end; mb += BMR) {
        if (mb + BMR < m_end) fetch(mb + BMR);
        if (DT == GNN_F32) {
            // half g of the wave owns tile rows g*16 .. g*16+15; step s multiplies row g*16+s
            const float* fA = (const float*)sA;
            const float* fD = (const float*)sD;
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                float av[MT], dv[NT];
#pragma unroll
                for (int i = 0; i < MT; ++i) av[i] = fA[(g * 16 + s) * A_LDW + wk * WTK + i * 32 + li];
#pragma unroll
                for (int j = 0; j < NT; ++j) dv[j] = fD[(g * 16 + s) * D_LDW + wn * WTN + j * 32 + li];
#pragma unroll
                for (int i = 0; i < MT; ++i)
#pragma unroll
                    for (int j = 0; j < NT; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], dv[j], acc[i][j], 0, 0, 0);
            }
        } else {
            // Step s (0, 1) multiplies tile rows s*16 + g*8 + e, e = 0..7: lane (li, g) needs those eight rows of
            // ONE column, and the tiles are row-major.  The LDS transpose read of gfx950 does that gather: in every
            // group of 16 lanes, lane 4e+q hands in the address of four consecutive columns (4q..4q+3) of row e and
            // lane j gets back column j of rows 0..3 (measured: result[j][e] = source[4e + j/4][j%4]).  Two reads
            // (rows +0..3, +4..7) make one operand.
            const int tl = lane & 15, tb = lane >> 4;              // lane within its group, group
            const int t_row = (tb >> 1) * 8 + (tl >> 2);           // g*8 + e
            const int t_col = (tb & 1) * 16 + (tl & 3) * 4;        // first of the four columns, inside the 32-column block
            const uint16_t* hA = (const uint16_t*)sA + t_row * (A_LDW * 2) + wk * WTK + t_col;
            const uint16_t* hD = (const uint16_t*)sD + t_row * (D_LDW * 2) + wn * WTN + t_col;
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                v8s av[MT], dv[NT];
#pragma unroll
                for (int i = 0; i < MT; ++i) {
                    const v4s lo = lds_tr16(hA + (s * 16) * (A_LDW * 2) + i * 32);
                    const v4s hi = lds_tr16(hA + (s * 16 + 4) * (A_LDW * 2) + i * 32);
                    av[i] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                }
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    const v4s lo = lds_tr16(hD + (s * 16) * (D_LDW * 2) + j * 32);
                    const v4s hi = lds_tr16(hD + (s * 16 + 4) * (D_LDW * 2) + j * 32);
                    dv[j] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                }
#pragma unroll
                for (int i = 0; i < MT; ++i)
#pragma unroll
                    for (int j = 0; j < NT; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, av[i]),
                                                                             __builtin_bit_cast(v8bf, dv[j]), acc[i][j], 0, 0, 0);
            }
        }
        __syncthreads();
        if (mb + BMR < m_end) {
            stash(mb + BMR);
            __syncthreads();
        }
    }

    if (do_bias) {   // uniform over the workgroup
#pragma unroll
        for (int c = 0; c < D_CH; ++c) {
            const int v = tid + 256 * c;
            if (v < BMR * D_VPR) {
#pragma unroll
                for (int e = 0; e < EPV; ++e) s_bs[v * EPV + e] = bs[c][e];
            }
        }
        __syncthreads();
        for (int col = tid; col < BN; col += 256) {
            float t = 0.f;
            for (int r = 0; r < BMR; ++r) t += s_bs[(r * D_VPR + col / EPV) * EPV + col % EPV];
            if (n0 + col < a.N) a.Pb[(int64_t)split * a.N + n0 + col] = t;
        }
    }
    float* P = a.P + ((int64_t)split * a.n_src + src) * (int64_t)a.K * a.N;
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int k = ko0 + wk * WTK + i * 32 + (r >> 2) * 8 + g * 4 + (r & 3);
            if (k >= a.K) continue;
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                const int n = n0 + wn * WTN + j * 32 + li;
                if (n < a.N) P[(int64_t)k * a.N + n] = acc[i][j][r];
            }
        }
}

// out_src[k][n] = sum over the row splits.  64 outputs x 4 split lanes per workgroup: lane y adds the splits y, y+4, ... in
// order and the four sums are added in lane order - a fixed tree (bit-reproducible) with four times the loads in flight
// of one chain over all splits (which took 72 us for 256 splits of a 128 x 256 gradient: as long as half the product).
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ P, int32_t splits, int32_t n_src,
                                                              int64_t kn, float* __restrict__ out0, float* __restrict__ out1) {
    __shared__ float s_sum[4][64];
    const int x = (int)(threadIdx.x & 63), y = (int)(threadIdx.x >> 6);
    const int64_t total = (int64_t)n_src * kn;
    for (int64_t base = (int64_t)blockIdx.x * 64; base < total; base += (int64_t)gridDim.x * 64) {   // uniform over the workgroup
        const int64_t i = base + x;
        float s = 0.f;
        if (i < total) {
#pragma unroll 8
            for (int32_t sp = y; sp < splits; sp += 4) s += P[(int64_t)sp * total + i];
        }
        s_sum[y][x] = s;
        __syncthreads();
        if (y == 0 && i < total) {
            const float t = ((s_sum[0][x] + s_sum[1][x]) + s_sum[2][x]) + s_sum[3][x];
            if (i < kn) out0[i] = t;
            else out1[i - kn] = t;
        }
        __syncthreads();
    }
}

// Wt[n][k] = W[k][n]; Wt rows are padded to ldt elements (pad left untouched, never read).
template <int DT>
__global__ __launch_bounds__(256) void transpose_kernel(const void* __restrict__ W, int32_t K, int32_t N, void* __restrict__ Wt,
                                                        int64_t ldt) {
    __shared__ uint32_t tile[32][33];
    const int k0 = blockIdx.x * 32, n0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    for (int r = ty; r < 32; r += 8) {
        const int k = k0 + r, n = n0 + tx;
        uint32_t v = 0;
        if (k < K && n < N) v = DT == GNN_F32 ? ((const uint32_t*)W)[(int64_t)k * N + n] : ((const uint16_t*)W)[(int64_t)k * N + n];
        tile[r][tx] = v;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const int n = n0 + r, k = k0 + tx;
        if (k < K && n < N) {
            if (DT == GNN_F32) ((uint32_t*)Wt)[(int64_t)n * ldt + k] = tile[tx][r];
            else ((uint16_t*)Wt)[(int64_t)n * ldt + k] = (uint16_t)tile[tx][r];
        }
    }
}

// dZ[i][0:N] = relu ? dH[row(i)] * [H[row(i)] > 0] : dH[row(i)], rows compacted (pad columns of dZ
// are written as zero; dZ == NULL: nothing is stored); column sums of each block of kDzRows rows go to part[block][0:N].
// Threads: cx 16-byte column vectors x 256/cx row lanes.
constexpr int kDzRows = 1024;

template <int DT>
__global__ __launch_bounds__(256) void dz_kernel(const int32_t* __restrict__ rows, int32_t M, const void* __restrict__ dH,
                                                 const void* __restrict__ H, int64_t ld_out, int32_t io_vec, int32_t relu,
                                                 int32_t N, void* __restrict__ dZ, int64_t ldz, float* __restrict__ part,
                                                 int32_t cx) {
    constexpr int EPV = DTy<DT>::EPV;
    __shared__ float s_sum[256 * EPV];
    const int tx = threadIdx.x % cx, ty = threadIdx.x / cx, ny = 256 / cx;
    const int64_t m_lo = (int64_t)blockIdx.x * kDzRows;
    const int64_t m_hi = m_lo + kDzRows < M ? m_lo + kDzRows : M;
    const int n_vec = (N + EPV - 1) / EPV;
    for (int vb = 0; vb < n_vec; vb += cx) {  // uniform trip count: the loop holds barriers
        const int n0 = (vb + tx) * EPV;
        float s[EPV];
#pragma unroll
        for (int e = 0; e < EPV; ++e) s[e] = 0.f;
        if (n0 < N) {
            for (int64_t m = m_lo + ty; m < m_hi; m += ny) {
                const int64_t r = rows ? (int64_t)rows[m] : m;
                const uint4 g4 = load16<DT>(dH, r * ld_out + n0, N - n0, io_vec != 0);
                uint4 h4 = make_uint4(0u, 0u, 0u, 0u);
                if (relu) h4 = load16<DT>(H, r * ld_out + n0, N - n0, io_vec != 0);
                uint4 o;
                if (DT == GNN_F32) {
                    float gv[4] = {__uint_as_float(g4.x), __uint_as_float(g4.y), __uint_as_float(g4.z), __uint_as_float(g4.w)};
                    const float hv[4] = {__uint_as_float(h4.x), __uint_as_float(h4.y), __uint_as_float(h4.z), __uint_as_float(h4.w)};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (relu && !(hv[e] > 0.f)) gv[e] = 0.f;
                        s[e] += gv[e];
                    }
                    o = make_uint4(__float_as_uint(gv[0]), __float_as_uint(gv[1]), __float_as_uint(gv[2]), __float_as_uint(gv[3]));
                } else {
                    // bf16 values pass through unchanged (or become 0), so the sum is over the stored values
                    const uint32_t gw[4] = {g4.x, g4.y, g4.z, g4.w};
                    const uint32_t hw[4] = {h4.x, h4.y, h4.z, h4.w};
                    uint32_t ow[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        uint32_t lo = gw[e] & 0xffffu, hi = gw[e] & 0xffff0000u;
                        if (relu && !(bf16lo(hw[e]) > 0.f)) lo = 0u;
                        if (relu && !(bf16hi(hw[e]) > 0.f)) hi = 0u;
                        s[2 * e] += __uint_as_float(lo << 16);
                        s[2 * e + 1] += __uint_as_float(hi);
                        ow[e] = lo | hi;
                    }
                    o = make_uint4(ow[0], ow[1], ow[2], ow[3]);
                }
                if (dZ == nullptr) continue;          // only the column sums are wanted
                if (DT == GNN_F32) *(uint4*)((float*)dZ + m * ldz + n0) = o;
                else *(uint4*)((uint16_t*)dZ + m * ldz + n0) = o;
            }
        }
#pragma unroll
        for (int e = 0; e < EPV; ++e) s_sum[(ty * cx + tx) * EPV + e] = s[e];
        __syncthreads();
        if (ty == 0 && n0 < N) {
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                float t = 0.f;
                for (int y = 0; y < ny; ++y) t += s_sum[(y * cx + tx) * EPV + e];
                if (n0 + e < N) part[(int64_t)blockIdx.x * N + n0 + e] = t;
            }
        }
        __syncthreads();
    }
}

// Wp[k][0:ldp] = W[k][0:N] followed by zeros: rows of an unaligned width become 16-byte aligned.
template <int DT>
__global__ __launch_bounds__(256) void pad_rows_kernel(const void* __restrict__ W, int32_t K, int32_t N, void* __restrict__ Wp, int32_t ldp) {
    const int64_t total = (int64_t)K * ldp;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int32_t k = (int32_t)(t / ldp), c = (int32_t)(t % ldp);
        if (DT == GNN_F32) ((float*)Wp)[t] = c < N ? ((const float*)W)[(int64_t)k * N + c] : 0.f;
        else ((uint16_t*)Wp)[t] = c < N ? ((const uint16_t*)W)[(int64_t)k * N + c] : (uint16_t)0;
    }
}

// out[n] = sum over the partial rows, in a fixed order: 32 row lanes x 32 columns per workgroup.
__global__ __launch_bounds__(1024) void reduce_rows_kernel(const float* __restrict__ part, int32_t n_blocks, int32_t N,
                                                           float* __restrict__ out) {
    __shared__ float s_sum[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int n = blockIdx.x * 32 + tx;
    float s = 0.f;
    if (n < N)
        for (int32_t b = ty; b < n_blocks; b += 32) s += part[(int64_t)b * N + n];
    s_sum[ty][tx] = s;
    __syncthreads();
    if (ty == 0 && n < N) {
        float t = 0.f;
#pragma unroll
        for (int y = 0; y < 32; ++y) t += s_sum[y][tx];
        out[n] = t;
    }
}

static inline bool vec_ok(const void* p, int64_t ld, int es) { return ((uintptr_t)p % 16 == 0) && ((ld * es) % 16 == 0); }

template <int DT>
static int32_t linear_fwd_impl(const int32_t* rows, int32_t n_active, const void* A, const void* Xs, int64_t ld_in, int32_t K,
                               const void* Wn, const void* Ws, const float* bias, int32_t N, void* H, int64_t ld_out,
                               int32_t relu, void* Wt0, void* Wt1, int64_t ldt, hipStream_t stream) {
    constexpr int ES = DTy<DT>::ES;
    dim3 tg((K + 31) / 32, (N + 31) / 32);
    transpose_kernel<DT><<<tg, 256, 0, stream>>>(Wn, K, N, Wt0, ldt);
    GNN_LAUNCH_CHECK("transpose_kernel");
    if (Xs) {
        transpose_kernel<DT><<<tg, 256, 0, stream>>>(Ws, K, N, Wt1, ldt);
        GNN_LAUNCH_CHECK("transpose_kernel");
    }
    GemmNT g;
    g.A[0] = A; g.A[1] = Xs; g.Bt[0] = Wt0; g.Bt[1] = Wt1; g.n_src = Xs ? 2 : 1;
    g.lda = ld_in; g.ldb = ldt;
    g.a_vec = vec_ok(A, ld_in, ES) && (!Xs || vec_ok(Xs, ld_in, ES));
    g.b_vec = 1;
    g.a_rows = rows; g.c_rows = rows; g.M = n_active; g.N = N; g.K = K;
    g.bias = bias; g.relu = relu; g.C = H; g.ldc = ld_out; g.c_vec = vec_ok(H, ld_out, ES);
    g.mask = nullptr; g.ldm = 0; g.m_vec = 0; g.n_acc = 0; g.M1 = INT32_MAX;
    return launch_gemm_nt<DT>(g, stream);
}

template <int DT>
static int32_t linear_bwd_impl(const int32_t* rows, int32_t M, const void* dH, const void* H, int64_t ld_out, int32_t relu,
                               const void* A, const void* Xs, int64_t ld_in, int32_t K, const void* Wn, const void* Ws, int32_t N,
                               float* dWn, float* dWs, float* dbias, void* dA, void* dXs, int64_t ld_din, void* dZ, int64_t ldz,
                               float* part, int32_t n_part, float* P, float* Pb, int32_t splits, int32_t rows_per_split,
                               void* Wpad0, void* Wpad1, int32_t ldwp, hipStream_t stream) {
    constexpr int ES = DTy<DT>::ES;
    // Without an activation to undo and without a row list, dH IS the compact dZ: no copy is made, the products read
    // dH in place and the weight-gradient kernel adds up the bias gradient on its way.
    const bool in_place = rows == nullptr && !relu && vec_ok(dH, ld_out, ES);
    if (in_place) {
        dZ = const_cast<void*>(dH);
        ldz = ld_out;
    } else {
        const int n_vec = (N + DTy<DT>::EPV - 1) / DTy<DT>::EPV;
        int cx = 4;
        while (cx < n_vec && cx < 256) cx <<= 1;
        const int io_vec = vec_ok(dH, ld_out, ES) && (!relu || vec_ok(H, ld_out, ES));
        dz_kernel<DT><<<n_part, 256, 0, stream>>>(rows, M, dH, H, ld_out, io_vec, relu, N, dZ, ldz, part, cx);
        GNN_LAUNCH_CHECK("dz_kernel");
        reduce_rows_kernel<<<(N + 31) / 32, 1024, 0, stream>>>(part, n_part, N, dbias);
        GNN_LAUNCH_CHECK("reduce_rows_kernel");
    }

    GemmTN t;
    t.A[0] = A; t.A[1] = Xs; t.n_src = Xs ? 2 : 1; t.lda = ld_in;
    t.a_vec = vec_ok(A, ld_in, ES) && (!Xs || vec_ok(Xs, ld_in, ES));
    t.a_rows = rows; t.D = dZ; t.ldd = ldz; t.d_vec = vec_ok(dZ, ldz, ES);
    t.M = M; t.N = N; t.K = K; t.rows_per_split = rows_per_split; t.n_splits = splits; t.P = P;
    t.Pb = in_place ? Pb : nullptr;
    const int ko_tiles = (K + 127) / 128;
    if (N > 32 && N <= 64) {      // class-score widths (41, 47): a 128-column tile would be two thirds padding
        const int64_t total = (int64_t)t.n_src * ko_tiles * splits;
        if (t.a_vec && t.d_vec) gemm_tn_kernel<DT, 64, true><<<(unsigned)((total + 7) / 8 * 8), 256, 0, stream>>>(t);
        else gemm_tn_kernel<DT, 64, false><<<(unsigned)((total + 7) / 8 * 8), 256, 0, stream>>>(t);
    } else if (tn_wide_columns(DT, N) && t.a_vec && t.d_vec) {
        if constexpr (DT == GNN_BF16) {
            const int64_t total = (int64_t)t.n_src * ko_tiles * (N / 256) * splits;
            gemm_tn_kernel<DT, 256, true><<<(unsigned)((total + 7) / 8 * 8), 256, 0, stream>>>(t);
        }
    } else if (N > 32) {
        const int64_t total = (int64_t)t.n_src * ko_tiles * ((N + 127) / 128) * splits;
        if (t.a_vec && t.d_vec) gemm_tn_kernel<DT, 128, true><<<(unsigned)((total + 7) / 8 * 8), 256, 0, stream>>>(t);
        else gemm_tn_kernel<DT, 128, false><<<(unsigned)((total + 7) / 8 * 8), 256, 0, stream>>>(t);
    } else {
        const int64_t total = (int64_t)t.n_src * ko_tiles * splits;
        if (t.a_vec && t.d_vec) gemm_tn_kernel<DT, 32, true><<<(unsigned)((total + 7) / 8 * 8), 256, 0, stream>>>(t);
        else gemm_tn_kernel<DT, 32, false><<<(unsigned)((total + 7) / 8 * 8), 256, 0, stream>>>(t);
    }
    GNN_LAUNCH_CHECK("gemm_tn_kernel");
    reduce_partials_kernel<<<grid_for((int64_t)t.n_src * K * N, 64, 8192), 256, 0, stream>>>(P, splits, t.n_src, (int64_t)K * N, dWn,
                                                                                           dWs);
    GNN_LAUNCH_CHECK("reduce_partials_kernel");
    if (in_place) {
        reduce_rows_kernel<<<(N + 31) / 32, 1024, 0, stream>>>(Pb, splits, N, dbias);
        GNN_LAUNCH_CHECK("reduce_rows_kernel");
    }

    // input gradients: dA = dZ W_neigh^T, dX_self = dZ W_self^T   (Bt = W as stored: [K][N])
    for (int which = 0; which < 2; ++which) {
        void* out = which == 0 ? dA : dXs;
        const void* W = which == 0 ? Wn : Ws;
        if (!out) continue;
        int64_t ldw = N;
        void* Wpad = which == 0 ? Wpad0 : Wpad1;
        if (Wpad != nullptr) {
            // rows of N elements are not 16-byte aligned (41 or 47 classes): the product reads a padded copy with vector loads
            pad_rows_kernel<DT><<<grid_for((int64_t)K * ldwp, 256, 1024), 256, 0, stream>>>(W, K, N, Wpad, ldwp);
            GNN_LAUNCH_CHECK("pad_rows_kernel");
            W = Wpad;
            ldw = ldwp;
        }
        GemmNT g;
        g.A[0] = dZ; g.A[1] = nullptr; g.Bt[0] = W; g.Bt[1] = nullptr; g.n_src = 1;
        g.lda = ldz; g.ldb = ldw; g.a_vec = vec_ok(dZ, ldz, ES); g.b_vec = vec_ok(W, ldw, ES);
        g.a_rows = nullptr; g.c_rows = rows; g.M = M; g.N = K; g.K = N;
        g.bias = nullptr; g.relu = 0; g.C = out; g.ldc = ld_din; g.c_vec = vec_ok(out, ld_din, ES);
        g.mask = nullptr; g.ldm = 0; g.m_vec = 0; g.n_acc = 0; g.M1 = INT32_MAX;
        GNN_CHECK(launch_gemm_nt<DT>(g, stream));
    }
    return GNN_OK;
}

static int32_t check_linear_common(int32_t n_active, int32_t K, int32_t N, int32_t dtype) {
    GNN_REQUIRE(n_active >= 0, GNN_ERR_INVALID_ARG, "negative row count");
    GNN_REQUIRE(dtype == GNN_F32 || dtype == GNN_BF16, GNN_ERR_UNSUPPORTED, "unknown dtype %d", dtype);
    GNN_REQUIRE(K >= 1 && N >= 1, GNN_ERR_INVALID_ARG, "K and N must be positive");
    GNN_REQUIRE(K <= kMaxDim && N <= kMaxDim, GNN_ERR_UNSUPPORTED, "K or N above %d", kMaxDim);
    return GNN_OK;
}

}  // namespace gnnhot

using namespace gnnhot;

extern "C" int32_t gnn_linear_fwd(const int32_t* rows, int32_t n_active, const void* A_neigh, const void* X_self, int64_t ld_in,
                                  int32_t K, const void* W_neigh, const void* W_self, const float* bias, int32_t N, void* H_out,
                                  int64_t ld_out, int32_t relu, int32_t dtype, void* ws, size_t* ws_bytes, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    GNN_CHECK(check_linear_common(n_active, K, N, dtype));
    GNN_REQUIRE(ld_in >= K && ld_out >= N, GNN_ERR_SHAPE, "leading dimension smaller than the width");
    GNN_REQUIRE((X_self == nullptr) == (W_self == nullptr), GNN_ERR_INVALID_ARG, "X_self and W_self must be given together");
    const int es = dtype == GNN_F32 ? 4 : 2;
    const int64_t ldt = (int64_t)align_up((size_t)K, 16 / es);
    WsCarver carve(ws);
    char* Wt0 = carve.take<char>((size_t)N * ldt * es);
    char* Wt1 = carve.take<char>((size_t)N * ldt * es);
    bool query;
    GNN_CHECK(ws_protocol(ws, ws_bytes, carve.used, &query));
    if (query) return GNN_OK;
    if (n_active == 0) return GNN_OK;
    GNN_REQUIRE(A_neigh && W_neigh && H_out, GNN_ERR_INVALID_ARG, "A_neigh, W_neigh or H_out is NULL");
    if (dtype == GNN_F32)
        return linear_fwd_impl<GNN_F32>(rows, n_active, A_neigh, X_self, ld_in, K, W_neigh, W_self, bias, N, H_out, ld_out, relu, Wt0,
                                        Wt1, ldt, stream);
    return linear_fwd_impl<GNN_BF16>(rows, n_active, A_neigh, X_self, ld_in, K, W_neigh, W_self, bias, N, H_out, ld_out, relu, Wt0,
                                     Wt1, ldt, stream);
}

// ---- the forward transform for callers that cannot allocate ---------------------------------
// Same kernels as gnn_linear_fwd; the two transposed weight copies live in a file-scope device array instead of a
// caller's workspace.  Every GPU holds its own copy of the array at its own address: the address is looked up once
// per device (with that device current) and only that pointer is ever handed to kernels.
constexpr size_t kStaticWtBytes = (size_t)4 << 20;   // one transposed weight matrix: N * round_up(K) elements
static __device__ __align__(256) unsigned char scratch[2 * kStaticWtBytes];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

static int32_t static_scratch(void** out) {
    int dev = -1;
    GNN_HIP(hipGetDevice(&dev));
    GNN_REQUIRE(dev >= 0 && dev < kMaxDevices, GNN_ERR_UNSUPPORTED, "device ordinal %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        GNN_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        GNN_REQUIRE(p != nullptr, GNN_ERR_HIP, "the scratch array has no address on device %d", dev);
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return GNN_OK;
}

extern "C" int32_t gnn_linear_fwd_static(const int32_t* rows, int32_t n_active, const void* A_neigh, const void* X_self,
                                         int64_t ld_in, int32_t K, const void* W_neigh, const void* W_self, const float* bias,
                                         int32_t N, void* H_out, int64_t ld_out, int32_t relu, int32_t dtype, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    GNN_CHECK(check_linear_common(n_active, K, N, dtype));
    GNN_REQUIRE(ld_in >= K && ld_out >= N, GNN_ERR_SHAPE, "leading dimension smaller than the width");
    GNN_REQUIRE((X_self == nullptr) == (W_self == nullptr), GNN_ERR_INVALID_ARG, "X_self and W_self must be given together");
    const int es = dtype == GNN_F32 ? 4 : 2;
    const int64_t ldt = (int64_t)align_up((size_t)K, 16 / es);
    const size_t wt_bytes = (size_t)N * ldt * es;
    GNN_REQUIRE(wt_bytes <= kStaticWtBytes, GNN_ERR_UNSUPPORTED,
                "weights of %d x %d elements of %d bytes need %zu bytes of scratch per matrix, the static array holds %zu: "
                "use gnn_linear_fwd with a workspace", K, N, es, wt_bytes, kStaticWtBytes);
    void* base = nullptr;
    GNN_CHECK(static_scratch(&base));     // also the set-up call: n_active == 0 resolves the address and returns
    if (n_active == 0) return GNN_OK;
    GNN_REQUIRE(A_neigh && W_neigh && H_out, GNN_ERR_INVALID_ARG, "A_neigh, W_neigh or H_out is NULL");
    char* Wt0 = (char*)base;
    char* Wt1 = (char*)base + kStaticWtBytes;
    if (dtype == GNN_F32)
        return linear_fwd_impl<GNN_F32>(rows, n_active, A_neigh, X_self, ld_in, K, W_neigh, W_self, bias, N, H_out, ld_out, relu, Wt0,
                                        Wt1, ldt, stream);
    return linear_fwd_impl<GNN_BF16>(rows, n_active, A_neigh, X_self, ld_in, K, W_neigh, W_self, bias, N, H_out, ld_out, relu, Wt0,
                                     Wt1, ldt, stream);
}

extern "C" int32_t gnn_linear_bwd(const int32_t* rows, int32_t n_active, const void* dH_out, const void* H_out, int64_t ld_out,
                                  int32_t relu, const void* A_neigh, const void* X_self, int64_t ld_in, int32_t K,
                                  const void* W_neigh, const void* W_self, int32_t N, float* dW_neigh, float* dW_self, float* dbias,
                                  void* dA_neigh, void* dX_self, int64_t ld_din, int32_t dtype, void* ws, size_t* ws_bytes,
                                  void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    GNN_CHECK(check_linear_common(n_active, K, N, dtype));
    GNN_REQUIRE(ld_in >= K && ld_out >= N, GNN_ERR_SHAPE, "leading dimension smaller than the width");
    GNN_REQUIRE((dA_neigh == nullptr && dX_self == nullptr) || ld_din >= K, GNN_ERR_SHAPE, "ld_din smaller than K");
    GNN_REQUIRE((X_self == nullptr) == (W_self == nullptr) && (X_self == nullptr) == (dW_self == nullptr), GNN_ERR_INVALID_ARG,
                "X_self, W_self and dW_self must be given together");
    GNN_REQUIRE(dX_self == nullptr || W_self != nullptr, GNN_ERR_INVALID_ARG, "dX_self needs W_self");
    const int es = dtype == GNN_F32 ? 4 : 2;
    const int n_src = X_self ? 2 : 1;
    const int64_t ldz = (int64_t)align_up((size_t)N, 16 / es);
    const int32_t n_part = n_active > 0 ? (n_active + kDzRows - 1) / kDzRows : 1;
    // Row splits of the weight-gradient reduction: as many as give every CU the three workgroups it can hold at once
    // and no more (256 CUs: 768 workgroups; the splits are equally long, so a second, partly filled round of workgroups
    // would cost a whole round: 1024 workgroups took 2 rounds where 768 take 1.33 of the old round's length), at least
    // 256 rows each, at most 256 splits and 128 MB of partial tiles
    const bool wide_n = tn_wide_columns(dtype, N) && vec_ok(A_neigh, ld_in, es) && (!X_self || vec_ok(X_self, ld_in, es));
    const int tiles = n_src * ((K + 127) / 128) * (wide_n ? N / 256 : (N > 32 ? (N + 127) / 128 : 1));
    int32_t splits = (wide_n ? 512 : 768) / tiles;   // two workgroups of the 256-column tile fit a CU, three of the others
    const int32_t max_splits = n_active > 0 ? (n_active + 255) / 256 : 1;
    const int64_t split_bytes = (int64_t)n_src * K * N * 4;
    if (splits > max_splits) splits = max_splits;
    if (splits > 256) splits = 256;
    if ((int64_t)splits * split_bytes > ((int64_t)128 << 20)) splits = (int32_t)(((int64_t)128 << 20) / split_bytes);
    if (splits < 1) splits = 1;
    int32_t rows_per_split = (int32_t)align_up((size_t)((n_active + splits - 1) / splits), 32);
    if (rows_per_split < 32) rows_per_split = 32;
    splits = n_active > 0 ? (n_active + rows_per_split - 1) / rows_per_split : 1;

    WsCarver carve(ws);
    char* dZ = carve.take<char>((size_t)(n_active > 0 ? n_active : 1) * ldz * es);
    float* part = carve.take<float>((size_t)n_part * N);
    float* P = carve.take<float>((size_t)splits * n_src * K * N);
    float* Pb = carve.take<float>((size_t)splits * N);
    // padded copies of the weights for the input-gradient products when a weight row is not a whole number of 16-byte vectors
    const bool pad_w = ((int64_t)N * es) % 16 != 0;
    const int32_t ldwp = (int32_t)ldz;
    char* Wpad0 = carve.take<char>(pad_w ? (size_t)K * ldwp * es : 0);
    char* Wpad1 = carve.take<char>(pad_w ? (size_t)K * ldwp * es : 0);
    if (!pad_w || ws == nullptr) Wpad0 = Wpad1 = nullptr;
    bool query;
    GNN_CHECK(ws_protocol(ws, ws_bytes, carve.used, &query));
    if (query) return GNN_OK;
    GNN_REQUIRE(dW_neigh && dbias, GNN_ERR_INVALID_ARG, "dW_neigh or dbias is NULL");
    if (n_active == 0) {
        fill_kernel<float><<<grid_for((int64_t)K * N, 256, 1024), 256, 0, stream>>>(dW_neigh, (int64_t)K * N, 0.f);
        if (dW_self) fill_kernel<float><<<grid_for((int64_t)K * N, 256, 1024), 256, 0, stream>>>(dW_self, (int64_t)K * N, 0.f);
        fill_kernel<float><<<1, 256, 0, stream>>>(dbias, (int64_t)N, 0.f);
        GNN_LAUNCH_CHECK("fill_kernel");
        return GNN_OK;
    }
    GNN_REQUIRE(dH_out && A_neigh && W_neigh, GNN_ERR_INVALID_ARG, "dH_out, A_neigh or W_neigh is NULL");
    GNN_REQUIRE(!relu || H_out, GNN_ERR_INVALID_ARG, "relu backward needs H_out");
    if (dtype == GNN_F32)
        return linear_bwd_impl<GNN_F32>(rows, n_active, dH_out, H_out, ld_out, relu, A_neigh, X_self, ld_in, K, W_neigh, W_self, N,
                                        dW_neigh, dW_self, dbias, dA_neigh, dX_self, ld_din, dZ, ldz, part, n_part, P, Pb, splits,
                                        rows_per_split, Wpad0, Wpad1, ldwp, stream);
    return linear_bwd_impl<GNN_BF16>(rows, n_active, dH_out, H_out, ld_out, relu, A_neigh, X_self, ld_in, K, W_neigh, W_self, N,
                                     dW_neigh, dW_self, dbias, dA_neigh, dX_self, ld_din, dZ, ldz, part, n_part, P, Pb, splits,
                                     rows_per_split, Wpad0, Wpad1, ldwp, stream);
}

extern "C" int32_t gnn_bias_grad(const int32_t* rows, int32_t n_active, const void* dZ, int64_t ldz, int32_t N, int32_t dtype,
                                 float* dbias, void* ws, size_t* ws_bytes, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    GNN_REQUIRE(n_active >= 0, GNN_ERR_INVALID_ARG, "negative row count");
    GNN_REQUIRE(dtype == GNN_F32 || dtype == GNN_BF16, GNN_ERR_UNSUPPORTED, "unknown dtype %d", dtype);
    GNN_REQUIRE(N >= 1 && N <= 4096, GNN_ERR_UNSUPPORTED, "N = %d out of range [1, 4096]", N);
    GNN_REQUIRE(ldz >= N, GNN_ERR_SHAPE, "leading dimension smaller than N = %d", N);
    const int32_t n_part = n_active > 0 ? (n_active + kDzRows - 1) / kDzRows : 1;
    WsCarver carve(ws);
    float* part = carve.take<float>((size_t)n_part * N);
    bool query;
    GNN_CHECK(ws_protocol(ws, ws_bytes, carve.used, &query));
    if (query) return GNN_OK;
    GNN_REQUIRE(dbias, GNN_ERR_INVALID_ARG, "dbias is NULL");
    if (n_active == 0) {
        fill_kernel<float><<<1, 256, 0, stream>>>(dbias, (int64_t)N, 0.f);
        GNN_LAUNCH_CHECK("fill_kernel");
        return GNN_OK;
    }
    GNN_REQUIRE(dZ, GNN_ERR_INVALID_ARG, "dZ is NULL");
    const int es = dtype == GNN_F32 ? 4 : 2, epv = 16 / es;
    const int n_vec = (N + epv - 1) / epv;
    int cx = 4;
    while (cx < n_vec && cx < 256) cx <<= 1;
    const int io_vec = ((uintptr_t)dZ % 16 == 0) && (ldz * es) % 16 == 0;
    if (dtype == GNN_F32) dz_kernel<GNN_F32><<<n_part, 256, 0, stream>>>(rows, n_active, dZ, nullptr, ldz, io_vec, 0, N, nullptr, 0, part, cx);
    else dz_kernel<GNN_BF16><<<n_part, 256, 0, stream>>>(rows, n_active, dZ, nullptr, ldz, io_vec, 0, N, nullptr, 0, part, cx);
    GNN_LAUNCH_CHECK("dz_kernel");
    reduce_rows_kernel<<<(N + 31) / 32, 1024, 0, stream>>>(part, n_part, N, dbias);
    GNN_LAUNCH_CHECK("reduce_rows_kernel");
    return GNN_OK;
}

extern "C" int32_t gnn_linear_bwd_input(const int32_t* rows, int32_t n_active, const void* dZ, int64_t lddz, int32_t N, const void* W,
                                        int32_t K, int32_t n_accumulate, const void* relu_H, int64_t ld_relu, void* dX, int64_t lddx,
                                        int32_t dtype, void* ws, size_t* ws_bytes, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    GNN_CHECK(check_linear_common(n_active, K, N, dtype));
    GNN_REQUIRE(lddz >= N && lddx >= K, GNN_ERR_SHAPE, "leading dimension smaller than the width");
    GNN_REQUIRE(n_accumulate >= 0 && n_accumulate <= n_active, GNN_ERR_INVALID_ARG, "n_accumulate = %d outside [0, n_active = %d]",
                n_accumulate, n_active);
    GNN_REQUIRE(relu_H == nullptr ? n_accumulate == 0 : ld_relu >= K, GNN_ERR_SHAPE,
                "relu_H: leading dimension smaller than K, or rows to accumulate without it");
    const int es = dtype == GNN_F32 ? 4 : 2;
    const bool pad_w = ((int64_t)N * es) % 16 != 0;
    const int32_t ldwp = (int32_t)align_up((size_t)N, 16 / es);
    WsCarver carve(ws);
    char* Wpad = carve.take<char>(pad_w ? (size_t)K * ldwp * es : 0);
    bool query;
    GNN_CHECK(ws_protocol(ws, ws_bytes, carve.used, &query));
    if (query) return GNN_OK;
    if (n_active == 0) return GNN_OK;
    GNN_REQUIRE(dZ && W && dX, GNN_ERR_INVALID_ARG, "dZ, W or dX is NULL");
    int64_t ldw = N;
    if (pad_w) {
        if (dtype == GNN_F32) pad_rows_kernel<GNN_F32><<<grid_for((int64_t)K * ldwp, 256, 1024), 256, 0, stream>>>(W, K, N, Wpad, ldwp);
        else pad_rows_kernel<GNN_BF16><<<grid_for((int64_t)K * ldwp, 256, 1024), 256, 0, stream>>>(W, K, N, Wpad, ldwp);
        GNN_LAUNCH_CHECK("pad_rows_kernel");
        W = Wpad;
        ldw = ldwp;
    }
    GemmNT g;
    g.A[0] = dZ; g.A[1] = nullptr; g.Bt[0] = W; g.Bt[1] = nullptr; g.n_src = 1;
    g.lda = lddz; g.ldb = ldw; g.a_vec = vec_ok(dZ, lddz, es); g.b_vec = vec_ok(W, ldw, es);
    g.a_rows = rows; g.c_rows = rows; g.M = n_active; g.N = K; g.K = N;
    g.bias = nullptr; g.relu = 0; g.C = dX; g.ldc = lddx; g.c_vec = vec_ok(dX, lddx, es);
    g.mask = relu_H; g.ldm = ld_relu; g.m_vec = relu_H ? vec_ok(relu_H, ld_relu, es) : 0; g.n_acc = n_accumulate; g.M1 = INT32_MAX;
    return dtype == GNN_F32 ? launch_gemm_nt<GNN_F32>(g, stream) : launch_gemm_nt<GNN_BF16>(g, stream);
}

extern "C" int32_t gnn_linear_bwd_input2(const int32_t* rows, int32_t n_active, const void* dG, const void* W_neigh, const void* dZ,
                                         const void* W_self, int32_t n_self, int64_t ldd, int32_t N, int32_t K, const void* relu_H,
                                         int64_t ld_relu, void* dX, int64_t lddx, int32_t dtype, void* ws, size_t* ws_bytes,
                                         void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    GNN_CHECK(check_linear_common(n_active, K, N, dtype));
    GNN_REQUIRE(ldd >= N && lddx >= K, GNN_ERR_SHAPE, "leading dimension smaller than the width");
    GNN_REQUIRE(n_self >= 0 && n_self <= n_active, GNN_ERR_INVALID_ARG, "n_self = %d outside [0, n_active = %d]", n_self, n_active);
    GNN_REQUIRE(relu_H == nullptr || ld_relu >= K, GNN_ERR_SHAPE, "relu_H: leading dimension smaller than K");
    const int es = dtype == GNN_F32 ? 4 : 2;
    const bool pad_w = ((int64_t)N * es) % 16 != 0;
    const int32_t ldwp = (int32_t)align_up((size_t)N, 16 / es);
    WsCarver carve(ws);
    char* Wpad0 = carve.take<char>(pad_w ? (size_t)K * ldwp * es : 0);
    char* Wpad1 = carve.take<char>(pad_w ? (size_t)K * ldwp * es : 0);
    bool query;
    GNN_CHECK(ws_protocol(ws, ws_bytes, carve.used, &query));
    if (query) return GNN_OK;
    if (n_active == 0) return GNN_OK;
    GNN_REQUIRE(dG && W_neigh && dX, GNN_ERR_INVALID_ARG, "dG, W_neigh or dX is NULL");
    GNN_REQUIRE(n_self == 0 || (dZ && W_self), GNN_ERR_INVALID_ARG, "dZ or W_self is NULL with n_self > 0");
    const bool two = n_self > 0;
    int64_t ldw = N;
    if (pad_w) {   // weight rows of an unaligned width (41 or 47 classes): the product reads padded copies with vector loads
        for (int which = 0; which < (two ? 2 : 1); ++which) {
            const void* W = which == 0 ? W_neigh : W_self;
            char* Wp = which == 0 ? Wpad0 : Wpad1;
            if (dtype == GNN_F32) pad_rows_kernel<GNN_F32><<<grid_for((int64_t)K * ldwp, 256, 1024), 256, 0, stream>>>(W, K, N, Wp, ldwp);
            else pad_rows_kernel<GNN_BF16><<<grid_for((int64_t)K * ldwp, 256, 1024), 256, 0, stream>>>(W, K, N, Wp, ldwp);
            GNN_LAUNCH_CHECK("pad_rows_kernel");
        }
        W_neigh = Wpad0;
        W_self = Wpad1;
        ldw = ldwp;
    }
    GemmNT g;
    g.A[0] = dG; g.A[1] = two ? dZ : nullptr; g.Bt[0] = W_neigh; g.Bt[1] = two ? W_self : nullptr; g.n_src = two ? 2 : 1;
    g.lda = ldd; g.ldb = ldw;
    g.a_vec = vec_ok(dG, ldd, es) && (!two || vec_ok(dZ, ldd, es));
    g.b_vec = vec_ok(W_neigh, ldw, es) && (!two || vec_ok(W_self, ldw, es));
    g.a_rows = rows; g.c_rows = rows; g.M = n_active; g.N = K; g.K = N;
    g.bias = nullptr; g.relu = 0; g.C = dX; g.ldc = lddx; g.c_vec = vec_ok(dX, lddx, es);
    g.mask = relu_H; g.ldm = ld_relu; g.m_vec = relu_H ? vec_ok(relu_H, ld_relu, es) : 0; g.n_acc = 0;
    g.M1 = two ? n_self : INT32_MAX;
    return dtype == GNN_F32 ? launch_gemm_nt<GNN_F32>(g, stream) : launch_gemm_nt<GNN_BF16>(g, stream);
}
