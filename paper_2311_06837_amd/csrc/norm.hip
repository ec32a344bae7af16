// Pre-activation of the deep residual GraphSAGE the paper trains (ResSAGE+, paper section 8.1; residual connections
// and pre-activation): t = ReLU(LayerNorm(x)) per vertex over its F features, its backward, and the residual add.
// A group of 8 to 64 lanes per row (16-byte vectors per lane when the rows are aligned; otherwise one wavefront per row
// with lane j on the columns j, j + 64, ...), F <= 1024: a row is read once into registers and the two statistics are
// reductions over the group.  Bound: HBM (2 row reads + 1 row write forward; 3-4 reads + 1 write backward).  The scale/shift
// gradients are summed per workgroup in a fixed order and then over the workgroups in a fixed order (no atomics).
#include "common.h"

namespace gnnhot {

constexpr int kLnMaxPerLane = 16;

template <int DT>
__device__ __forceinline__ float ln_load(const void* p, int64_t off) {
    if (DT == GNN_F32) return ((const float*)p)[off];
    return bf16_to_f32(((const uint16_t*)p)[off]);
}
template <int DT>
__device__ __forceinline__ void ln_store(void* p, int64_t off, float v) {
    if (DT == GNN_F32) ((float*)p)[off] = v;
    else ((uint16_t*)p)[off] = f32_to_bf16(v);
}
__device__ __forceinline__ float ln_wave_sum(float x) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, kWave);
    return x;
}

// ---- vector route: 16-byte aligned rows --------------------------------------------------------------------------
// LR lanes (8 .. 64) own a row, 64 / LR rows share a wavefront; lane sl holds the 16-byte vectors sl, sl + LR, ... of
// its row (NV of them), so a row is one or a few fully coalesced loads and the statistics are reductions over LR lanes.
template <int DT>
struct LnVec {
    static constexpr int VE = DT == GNN_F32 ? 4 : 8;
    static __device__ __forceinline__ void load(const void* p, int64_t elem_off, float (&out)[VE]) {
        const uint4 r = *(const uint4*)((const char*)p + elem_off * (DT == GNN_F32 ? 4 : 2));
        if (DT == GNN_F32) {
            out[0] = __uint_as_float(r.x); out[1] = __uint_as_float(r.y); out[2] = __uint_as_float(r.z); out[3] = __uint_as_float(r.w);
        } else {
            const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                out[2 * e] = bf16lo(w[e]);
                out[2 * e + 1] = bf16hi(w[e]);
            }
        }
    }
    // stores the first n_valid elements (a full vector as one 16-byte store)
    static __device__ __forceinline__ void store(void* p, int64_t elem_off, const float (&v)[VE], int n_valid) {
        if (n_valid >= VE) {
            uint4 r;
            if (DT == GNN_F32) {
                r = make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
            } else {
                r = make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]));
            }
            *(uint4*)((char*)p + elem_off * (DT == GNN_F32 ? 4 : 2)) = r;
        } else {
            for (int e = 0; e < n_valid; ++e) ln_store<DT>(p, elem_off + e, v[e]);
        }
    }
};

template <int LR>
__device__ __forceinline__ float ln_group_sum(float x) {
#pragma unroll
    for (int d = LR / 2; d >= 1; d >>= 1) x += __shfl_xor(x, d, kWave);
    return x;
}

template <int DT, int LR, int NV>
__global__ __launch_bounds__(256) void ln_relu_fwd_vec_kernel(const int32_t* __restrict__ rows, int32_t n_active, const void* __restrict__ X,
                                                              int64_t ldx, int32_t F, const float* __restrict__ gamma,
                                                              const float* __restrict__ beta, float eps, void* __restrict__ Y, int64_t ldy) {
    constexpr int VE = LnVec<DT>::VE, RPW = 64 / LR;
    const int lane = lane_id(), sub = lane / LR, sl = lane % LR;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6, n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const float inv_f = 1.0f / (float)F;
    float gm[NV][VE], bt[NV][VE];   // the lane's share of scale and shift, read once
#pragma unroll
    for (int k = 0; k < NV; ++k)
#pragma unroll
        for (int e = 0; e < VE; ++e) {
            const int c = (sl + LR * k) * VE + e;
            gm[k][e] = c < F ? gamma[c] : 0.f;
            bt[k][e] = c < F ? beta[c] : 0.f;
        }
    for (int64_t base = wave * RPW; base < n_active; base += n_waves * RPW) {   // uniform over the wavefront
        const int64_t i = base + sub;
        const bool active = i < n_active;
        const int64_t v = active ? (rows ? (int64_t)rows[i] : i) : 0;
        float x[NV][VE];
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int c0 = (sl + LR * k) * VE;
            if (active && c0 < F) LnVec<DT>::load(X, v * ldx + c0, x[k]);
#pragma unroll
            for (int e = 0; e < VE; ++e) {
                if (!(active && c0 + e < F)) x[k][e] = 0.f;
                s += x[k][e];
            }
        }
        const float mu = ln_group_sum<LR>(s) * inv_f;
        float q = 0.f;
#pragma unroll
        for (int k = 0; k < NV; ++k)
#pragma unroll
            for (int e = 0; e < VE; ++e) {
                const float d = (sl + LR * k) * VE + e < F ? x[k][e] - mu : 0.f;
                q += d * d;
            }
        const float rstd = 1.0f / sqrtf(ln_group_sum<LR>(q) * inv_f + eps);
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int c0 = (sl + LR * k) * VE;
            if (active && c0 < F) {
                float o[VE];
#pragma unroll
                for (int e = 0; e < VE; ++e) {
                    const float t = (x[k][e] - mu) * rstd * gm[k][e] + bt[k][e];
                    o[e] = t > 0.f ? t : 0.f;
                }
                LnVec<DT>::store(Y, v * ldy + c0, o, F - c0);
            }
        }
    }
}

constexpr int kLnVecRowsPerBlock = 256;

// dX[v] = LN-backward(dY[v] where T[v] > 0) (+ dRes[v] for the first n_res listed rows: the residual connection);
// part[block][0:F] = sum over the block's rows of g * xhat, part[block][F:2F] = sum of g (lane groups in a fixed
// pattern, added in a fixed order).
template <int DT, int LR, int NV>
__global__ __launch_bounds__(256) void ln_relu_bwd_vec_kernel(const int32_t* __restrict__ rows, int32_t n_active, const void* __restrict__ dY,
                                                              int64_t lddy, const void* __restrict__ T, int64_t ldt,
                                                              const void* __restrict__ X, int64_t ldx, int32_t F,
                                                              const float* __restrict__ gamma, float eps, const void* __restrict__ dRes,
                                                              int64_t ldr, int32_t n_res, void* __restrict__ dX, int64_t lddx,
                                                              float* __restrict__ part) {
    constexpr int VE = LnVec<DT>::VE, GROUPS = 256 / LR, COLS = LR * NV * VE;
    __shared__ float s_g[GROUPS * COLS], s_b[GROUPS * COLS];
    const int grp = (int)threadIdx.x / LR, sl = (int)threadIdx.x % LR;
    const float inv_f = 1.0f / (float)F;
    float ag[NV][VE], ab[NV][VE], gm[NV][VE];
#pragma unroll
    for (int k = 0; k < NV; ++k)
#pragma unroll
        for (int e = 0; e < VE; ++e) {
            ag[k][e] = ab[k][e] = 0.f;
            const int c = (sl + LR * k) * VE + e;
            gm[k][e] = c < F ? gamma[c] : 0.f;
        }
    const int64_t r0 = (int64_t)blockIdx.x * kLnVecRowsPerBlock;
    for (int r = 0; r < kLnVecRowsPerBlock; r += GROUPS) {          // uniform over the workgroup
        const int64_t i = r0 + r + grp;
        const bool active = i < n_active;
        const int64_t v = active ? (rows ? (int64_t)rows[i] : i) : 0;
        float x[NV][VE], g[NV][VE];
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int c0 = (sl + LR * k) * VE;
            float t[VE];
            const bool ok = active && c0 < F;
            if (ok) {
                LnVec<DT>::load(X, v * ldx + c0, x[k]);
                LnVec<DT>::load(dY, v * lddy + c0, g[k]);
                LnVec<DT>::load(T, v * ldt + c0, t);
            }
#pragma unroll
            for (int e = 0; e < VE; ++e) {
                const bool in = ok && c0 + e < F;
                x[k][e] = in ? x[k][e] : 0.f;
                g[k][e] = (in && t[e] > 0.f) ? g[k][e] : 0.f;
                s += x[k][e];
            }
        }
        const float mu = ln_group_sum<LR>(s) * inv_f;
        float q = 0.f;
#pragma unroll
        for (int k = 0; k < NV; ++k)
#pragma unroll
            for (int e = 0; e < VE; ++e) {
                const float d = (sl + LR * k) * VE + e < F ? x[k][e] - mu : 0.f;
                q += d * d;
            }
        const float rstd = 1.0f / sqrtf(ln_group_sum<LR>(q) * inv_f + eps);
        float m1 = 0.f, m2 = 0.f;
#pragma unroll
        for (int k = 0; k < NV; ++k)
#pragma unroll
            for (int e = 0; e < VE; ++e) {
                const bool in = (sl + LR * k) * VE + e < F;
                x[k][e] = in ? (x[k][e] - mu) * rstd : 0.f;       // xhat
                ag[k][e] += g[k][e] * x[k][e];
                ab[k][e] += g[k][e];
                g[k][e] *= gm[k][e];
                m1 += g[k][e];
                m2 += g[k][e] * x[k][e];
            }
        m1 = ln_group_sum<LR>(m1) * inv_f;
        m2 = ln_group_sum<LR>(m2) * inv_f;
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int c0 = (sl + LR * k) * VE;
            if (active && c0 < F) {
                float o[VE];
#pragma unroll
                for (int e = 0; e < VE; ++e) o[e] = rstd * (g[k][e] - m1 - x[k][e] * m2);
                if (dRes != nullptr && i < n_res) {
                    float rr[VE];
                    LnVec<DT>::load(dRes, v * ldr + c0, rr);
#pragma unroll
                    for (int e = 0; e < VE; ++e) o[e] += c0 + e < F ? rr[e] : 0.f;
                }
                LnVec<DT>::store(dX, v * lddx + c0, o, F - c0);
            }
        }
    }
#pragma unroll
    for (int k = 0; k < NV; ++k)
#pragma unroll
        for (int e = 0; e < VE; ++e) {
            s_g[grp * COLS + (sl + LR * k) * VE + e] = ag[k][e];
            s_b[grp * COLS + (sl + LR * k) * VE + e] = ab[k][e];
        }
    __syncthreads();
    for (int c = threadIdx.x; c < F; c += 256) {
        float tg = 0.f, tb = 0.f;
        for (int q = 0; q < GROUPS; ++q) {
            tg += s_g[q * COLS + c];
            tb += s_b[q * COLS + c];
        }
        part[(int64_t)blockIdx.x * 2 * F + c] = tg;
        part[(int64_t)blockIdx.x * 2 * F + F + c] = tb;
    }
}

// ---- element route: any alignment; lane j owns the columns j, j + 64, ... (NJ of them) ------------------------
template <int DT, int NJ>
__global__ __launch_bounds__(256) void ln_relu_fwd_kernel(const int32_t* __restrict__ rows, int32_t n_active, const void* __restrict__ X,
                                                          int64_t ldx, int32_t F, const float* __restrict__ gamma,
                                                          const float* __restrict__ beta, float eps, void* __restrict__ Y, int64_t ldy) {
    const int lane = lane_id();
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6, n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const float inv_f = 1.0f / (float)F;
    for (int64_t i = wave; i < n_active; i += n_waves) {
        const int64_t v = rows ? (int64_t)rows[i] : i;
        float x[NJ];
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int c = lane + 64 * j;
            x[j] = c < F ? ln_load<DT>(X, v * ldx + c) : 0.f;
            s += x[j];
        }
        const float mu = ln_wave_sum(s) * inv_f;
        float q = 0.f;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int c = lane + 64 * j;
            const float d = c < F ? x[j] - mu : 0.f;
            q += d * d;
        }
        const float rstd = 1.0f / sqrtf(ln_wave_sum(q) * inv_f + eps);
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int c = lane + 64 * j;
            if (c < F) {
                const float t = (x[j] - mu) * rstd * gamma[c] + beta[c];
                ln_store<DT>(Y, v * ldy + c, t > 0.f ? t : 0.f);
            }
        }
    }
}

template <int DT, int NJ>
__global__ __launch_bounds__(256) void ln_relu_bwd_kernel(const int32_t* __restrict__ rows, int32_t n_active, const void* __restrict__ dY,
                                                          int64_t lddy, const void* __restrict__ T, int64_t ldt,
                                                          const void* __restrict__ X, int64_t ldx, int32_t F,
                                                          const float* __restrict__ gamma, float eps, const void* __restrict__ dRes,
                                                          int64_t ldr, int32_t n_res, void* __restrict__ dX, int64_t lddx,
                                                          float* __restrict__ part) {
    __shared__ float s_g[4][NJ * 64], s_b[4][NJ * 64];
    const int lane = lane_id(), wave = (int)(threadIdx.x >> 6);
    const float inv_f = 1.0f / (float)F;
    float ag[NJ], ab[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) ag[j] = ab[j] = 0.f;
    const int64_t r0 = (int64_t)blockIdx.x * kLnVecRowsPerBlock;
    for (int k = wave; k < kLnVecRowsPerBlock; k += 4) {     // fixed assignment of rows to waves
        const int64_t i = r0 + k;
        if (i >= n_active) break;                            // uniform over the wave
        const int64_t v = rows ? (int64_t)rows[i] : i;
        float x[NJ], g[NJ];
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int c = lane + 64 * j;
            x[j] = c < F ? ln_load<DT>(X, v * ldx + c) : 0.f;
            s += x[j];
        }
        const float mu = ln_wave_sum(s) * inv_f;
        float q = 0.f;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int c = lane + 64 * j;
            const float d = c < F ? x[j] - mu : 0.f;
            q += d * d;
        }
        const float rstd = 1.0f / sqrtf(ln_wave_sum(q) * inv_f + eps);
        float m1 = 0.f, m2 = 0.f;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int c = lane + 64 * j;
            float gv = 0.f;
            if (c < F) {
                x[j] = (x[j] - mu) * rstd;                   // xhat
                gv = ln_load<DT>(T, v * ldt + c) > 0.f ? ln_load<DT>(dY, v * lddy + c) : 0.f;
                ag[j] += gv * x[j];
                ab[j] += gv;
                gv *= gamma[c];
            } else {
                x[j] = 0.f;
            }
            g[j] = gv;
            m1 += gv;
            m2 += gv * x[j];
        }
        m1 = ln_wave_sum(m1) * inv_f;
        m2 = ln_wave_sum(m2) * inv_f;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int c = lane + 64 * j;
            if (c < F) {
                float o = rstd * (g[j] - m1 - x[j] * m2);
                if (dRes != nullptr && i < n_res) o += ln_load<DT>(dRes, v * ldr + c);
                ln_store<DT>(dX, v * lddx + c, o);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        s_g[wave][lane + 64 * j] = ag[j];
        s_b[wave][lane + 64 * j] = ab[j];
    }
    __syncthreads();
    for (int c = threadIdx.x; c < F; c += 256) {
        part[(int64_t)blockIdx.x * 2 * F + c] = (s_g[0][c] + s_g[1][c]) + (s_g[2][c] + s_g[3][c]);
        part[(int64_t)blockIdx.x * 2 * F + F + c] = (s_b[0][c] + s_b[1][c]) + (s_b[2][c] + s_b[3][c]);
    }
}

// out0[c] = sum_b part[b][c], out1[c] = sum_b part[b][F + c], blocks in order: 32 row lanes x 32 columns per workgroup
__global__ __launch_bounds__(1024) void ln_reduce_kernel(const float* __restrict__ part, int32_t n_blocks, int32_t F, float* __restrict__ out0,
                                                         float* __restrict__ out1) {
    __shared__ float s_sum[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int c = blockIdx.x * 32 + tx;   // column of the [n_blocks][2F] matrix
    float s = 0.f;
    if (c < 2 * F)
        for (int32_t b = ty; b < n_blocks; b += 32) s += part[(int64_t)b * 2 * F + c];
    s_sum[ty][tx] = s;
    __syncthreads();
    if (ty == 0 && c < 2 * F) {
        float t = 0.f;
#pragma unroll
        for (int y = 0; y < 32; ++y) t += s_sum[y][tx];
        if (c < F) out0[c] = t;
        else out1[c - F] = t;
    }
}

// Y[v, 0:F] += X[v, 0:F] for the listed rows (the residual connection, forward).  Only the first n_add listed rows take
// the addition; with H (nullable, same rows and columns as Y) what is stored is zeroed where H <= 0 - for every listed
// row.  VEC: 16-byte aligned rows and F a multiple of the vector - a lane adds one 16-byte vector, consecutive lanes walk
// along the row and on to the next rows.
template <int DT, bool VEC>
__global__ __launch_bounds__(256) void add_rows_kernel(const int32_t* __restrict__ rows, int32_t n_active, const void* __restrict__ X,
                                                       int64_t ldx, int32_t n_add, void* __restrict__ Y, int64_t ldy, int32_t F,
                                                       const void* __restrict__ H, int64_t ldh) {
    if (VEC) {
        // a thread keeps its column vector and walks down the rows: the workgroup covers `rb` rows x `vpr` vectors at a
        // time (or, for rows of more than 256 vectors, one row in several sweeps) - no division inside the loop
        constexpr int VE = LnVec<DT>::VE;
        const int vpr = F / VE;
        const int rb = vpr < 256 ? 256 / vpr : 1;
        const int r0 = vpr < 256 ? (int)threadIdx.x / vpr : 0;
        const int cstart = vpr < 256 ? (int)threadIdx.x % vpr : (int)threadIdx.x;
        if (r0 >= rb) return;
        for (int64_t i = (int64_t)blockIdx.x * rb + r0; i < n_active; i += (int64_t)gridDim.x * rb) {
            const int64_t v = rows ? (int64_t)rows[i] : i;
            for (int cv = cstart; cv < vpr; cv += 256) {
                const int c0 = cv * VE;
                float a[VE], b[VE];
                LnVec<DT>::load(Y, v * ldy + c0, a);
                if (i < n_add) {
                    LnVec<DT>::load(X, v * ldx + c0, b);
#pragma unroll
                    for (int e = 0; e < VE; ++e) a[e] += b[e];
                }
                if (H) {
                    LnVec<DT>::load(H, v * ldh + c0, b);
#pragma unroll
                    for (int e = 0; e < VE; ++e) a[e] = b[e] > 0.f ? a[e] : 0.f;
                }
                LnVec<DT>::store(Y, v * ldy + c0, a, VE);
            }
        }
        return;
    }
    const int lane = lane_id();
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6, n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t i = wave; i < n_active; i += n_waves) {
        const int64_t v = rows ? (int64_t)rows[i] : i;
        for (int c = lane; c < F; c += 64) {
            float a = ln_load<DT>(Y, v * ldy + c);
            if (i < n_add) a += ln_load<DT>(X, v * ldx + c);
            if (H && !(ln_load<DT>(H, v * ldh + c) > 0.f)) a = 0.f;
            ln_store<DT>(Y, v * ldy + c, a);
        }
    }
}

static int32_t ln_check(int32_t n_active, int32_t F, int32_t dtype) {
    GNN_REQUIRE(n_active >= 0, GNN_ERR_INVALID_ARG, "negative row count");
    GNN_REQUIRE(dtype == GNN_F32 || dtype == GNN_BF16, GNN_ERR_UNSUPPORTED, "unknown dtype %d", dtype);
    GNN_REQUIRE(F >= 1 && F <= 64 * kLnMaxPerLane, GNN_ERR_UNSUPPORTED, "F = %d out of range [1, %d]", F, 64 * kLnMaxPerLane);
    return GNN_OK;
}

}  // namespace gnnhot

using namespace gnnhot;

extern "C" int32_t gnn_layer_norm_relu_fwd(const int32_t* rows, int32_t n_active, const void* X, int64_t ldx, int32_t F,
                                           const float* gamma, const float* beta, float eps, void* Y, int64_t ldy, int32_t dtype,
                                           void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    GNN_CHECK(ln_check(n_active, F, dtype));
    GNN_REQUIRE(ldx >= F && ldy >= F, GNN_ERR_SHAPE, "leading dimension smaller than F = %d", F);
    if (n_active == 0) return GNN_OK;
    GNN_REQUIRE(X && Y && gamma && beta, GNN_ERR_INVALID_ARG, "X, Y, gamma or beta is NULL");
    const int es = dtype == GNN_F32 ? 4 : 2, ve = 16 / es;
    const bool vec = ((uintptr_t)X % 16 == 0) && ((uintptr_t)Y % 16 == 0) && (ldx * es) % 16 == 0 && (ldy * es) % 16 == 0;
    const int n_vec = (F + ve - 1) / ve;
#define GNN_LN_FWD_V(DT_, LR_, NV_)                                                                                        \
    ln_relu_fwd_vec_kernel<DT_, LR_, NV_><<<grid_for((int64_t)n_active * LR_, 256, 1 << 14), 256, 0, stream>>>(rows, n_active, X, ldx, F, gamma, \
                                                                                                           beta, eps, Y, ldy)
#define GNN_LN_FWD_S(DT_, NJ_)                                                                                             \
    ln_relu_fwd_kernel<DT_, NJ_><<<grid_for((int64_t)n_active * 64, 256, 1 << 14), 256, 0, stream>>>(rows, n_active, X, ldx, F, gamma, beta, \
                                                                                                 eps, Y, ldy)
#define GNN_LN_FWD(DT_)                                    \
    if (vec && n_vec <= 8) GNN_LN_FWD_V(DT_, 8, 1);        \
    else if (vec && n_vec <= 16) GNN_LN_FWD_V(DT_, 16, 1); \
    else if (vec && n_vec <= 32) GNN_LN_FWD_V(DT_, 32, 1); \
    else if (vec && n_vec <= 64) GNN_LN_FWD_V(DT_, 64, 1); \
    else if (vec && n_vec <= 128) GNN_LN_FWD_V(DT_, 64, 2);\
    else if (vec && DT_ == GNN_F32) GNN_LN_FWD_V(GNN_F32, 64, 4); \
    else if (F <= 128) GNN_LN_FWD_S(DT_, 2);               \
    else if (F <= 256) GNN_LN_FWD_S(DT_, 4);               \
    else GNN_LN_FWD_S(DT_, 16);
    if (dtype == GNN_F32) { GNN_LN_FWD(GNN_F32) } else { GNN_LN_FWD(GNN_BF16) }
#undef GNN_LN_FWD
#undef GNN_LN_FWD_V
#undef GNN_LN_FWD_S
    GNN_LAUNCH_CHECK("ln_relu_fwd_kernel");
    return GNN_OK;
}

extern "C" int32_t gnn_layer_norm_relu_bwd(const int32_t* rows, int32_t n_active, const void* dY, int64_t lddy, const void* T, int64_t ldt,
                                           const void* X, int64_t ldx, int32_t F, const float* gamma, float eps, const void* dRes,
                                           int64_t ldr, int32_t n_res, void* dX, int64_t lddx, float* dgamma, float* dbeta,
                                           int32_t dtype, void* ws, size_t* ws_bytes, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    GNN_CHECK(ln_check(n_active, F, dtype));
    GNN_REQUIRE(lddy >= F && ldt >= F && ldx >= F && lddx >= F && (dRes == nullptr || ldr >= F), GNN_ERR_SHAPE,
                "leading dimension smaller than F = %d", F);
    GNN_REQUIRE(n_res >= 0 && n_res <= n_active, GNN_ERR_INVALID_ARG, "n_res out of range");
    const int32_t n_blocks = n_active > 0 ? (n_active + kLnVecRowsPerBlock - 1) / kLnVecRowsPerBlock : 1;
    WsCarver carve(ws);
    float* part = carve.take<float>((size_t)n_blocks * 2 * F);
    bool query;
    GNN_CHECK(ws_protocol(ws, ws_bytes, carve.used, &query));
    if (query) return GNN_OK;
    GNN_REQUIRE(dgamma && dbeta, GNN_ERR_INVALID_ARG, "dgamma or dbeta is NULL");
    if (n_active == 0) {
        fill_kernel<float><<<1, 256, 0, stream>>>(dgamma, (int64_t)F, 0.f);
        fill_kernel<float><<<1, 256, 0, stream>>>(dbeta, (int64_t)F, 0.f);
        GNN_LAUNCH_CHECK("fill_kernel");
        return GNN_OK;
    }
    GNN_REQUIRE(dY && T && X && dX && gamma, GNN_ERR_INVALID_ARG, "dY, T, X, dX or gamma is NULL");
    const int es = dtype == GNN_F32 ? 4 : 2, ve = 16 / es;
    auto al = [&](const void* p, int64_t ld) { return ((uintptr_t)p % 16 == 0) && (ld * es) % 16 == 0; };
    const bool vec = al(dY, lddy) && al(T, ldt) && al(X, ldx) && al(dX, lddx) && (dRes == nullptr || al(dRes, ldr));
    const int n_vec = (F + ve - 1) / ve;
#define GNN_LN_ARGS rows, n_active, dY, lddy, T, ldt, X, ldx, F, gamma, eps, dRes, ldr, n_res, dX, lddx, part
#define GNN_LN_BWD(DT_)                                                                                     \
    if (vec && n_vec <= 8) ln_relu_bwd_vec_kernel<DT_, 8, 1><<<n_blocks, 256, 0, stream>>>(GNN_LN_ARGS);     \
    else if (vec && n_vec <= 16) ln_relu_bwd_vec_kernel<DT_, 16, 1><<<n_blocks, 256, 0, stream>>>(GNN_LN_ARGS); \
    else if (vec && n_vec <= 32) ln_relu_bwd_vec_kernel<DT_, 32, 1><<<n_blocks, 256, 0, stream>>>(GNN_LN_ARGS); \
    else if (vec && n_vec <= 64) ln_relu_bwd_vec_kernel<DT_, 64, 1><<<n_blocks, 256, 0, stream>>>(GNN_LN_ARGS); \
    else if (vec && n_vec <= 128) ln_relu_bwd_vec_kernel<DT_, 64, 2><<<n_blocks, 256, 0, stream>>>(GNN_LN_ARGS); \
    else if (vec && DT_ == GNN_F32) ln_relu_bwd_vec_kernel<GNN_F32, 64, 4><<<n_blocks, 256, 0, stream>>>(GNN_LN_ARGS); \
    else if (F <= 128) ln_relu_bwd_kernel<DT_, 2><<<n_blocks, 256, 0, stream>>>(GNN_LN_ARGS);                \
    else if (F <= 256) ln_relu_bwd_kernel<DT_, 4><<<n_blocks, 256, 0, stream>>>(GNN_LN_ARGS);                \
    else ln_relu_bwd_kernel<DT_, 16><<<n_blocks, 256, 0, stream>>>(GNN_LN_ARGS);
    if (dtype == GNN_F32) { GNN_LN_BWD(GNN_F32) } else { GNN_LN_BWD(GNN_BF16) }
#undef GNN_LN_BWD
#undef GNN_LN_ARGS
    GNN_LAUNCH_CHECK("ln_relu_bwd_kernel");
    ln_reduce_kernel<<<(2 * F + 31) / 32, 1024, 0, stream>>>(part, n_blocks, F, dgamma, dbeta);
    GNN_LAUNCH_CHECK("ln_reduce_kernel");
    return GNN_OK;
}

static int32_t add_rows_impl(const int32_t* rows, int32_t n_active, const void* X, int64_t ldx, int32_t n_add, void* Y, int64_t ldy,
                             int32_t F, const void* H, int64_t ldh, int32_t dtype, hipStream_t stream) {
    GNN_REQUIRE(n_active >= 0 && F >= 0, GNN_ERR_INVALID_ARG, "negative size");
    GNN_REQUIRE(n_add >= 0 && n_add <= n_active, GNN_ERR_INVALID_ARG, "n_add = %d outside [0, n_active = %d]", n_add, n_active);
    GNN_REQUIRE(dtype == GNN_F32 || dtype == GNN_BF16, GNN_ERR_UNSUPPORTED, "unknown dtype %d", dtype);
    GNN_REQUIRE((n_add == 0 || ldx >= F) && ldy >= F && (H == nullptr || ldh >= F), GNN_ERR_SHAPE, "leading dimension smaller than F = %d", F);
    if (n_active == 0 || F == 0) return GNN_OK;
    GNN_REQUIRE((X || n_add == 0) && Y, GNN_ERR_INVALID_ARG, "X or Y is NULL");
    const int es = dtype == GNN_F32 ? 4 : 2, ve = 16 / es;
    const bool vec = (n_add == 0 || ((uintptr_t)X % 16 == 0 && (ldx * es) % 16 == 0)) && ((uintptr_t)Y % 16 == 0) && (ldy * es) % 16 == 0 &&
                     (H == nullptr || ((uintptr_t)H % 16 == 0 && (ldh * es) % 16 == 0)) && F % ve == 0;
    const int vpr = F / ve, rb = (vec && vpr < 256) ? 256 / vpr : 1;       // rows one workgroup covers per sweep (vector route)
    const int grid = vec ? grid_for(((int64_t)n_active + rb - 1) / rb * 256, 256, 1 << 14) : grid_for((int64_t)n_active * 64, 256, 1 << 14);
    if (dtype == GNN_F32) {
        if (vec) add_rows_kernel<GNN_F32, true><<<grid, 256, 0, stream>>>(rows, n_active, X, ldx, n_add, Y, ldy, F, H, ldh);
        else add_rows_kernel<GNN_F32, false><<<grid, 256, 0, stream>>>(rows, n_active, X, ldx, n_add, Y, ldy, F, H, ldh);
    } else {
        if (vec) add_rows_kernel<GNN_BF16, true><<<grid, 256, 0, stream>>>(rows, n_active, X, ldx, n_add, Y, ldy, F, H, ldh);
        else add_rows_kernel<GNN_BF16, false><<<grid, 256, 0, stream>>>(rows, n_active, X, ldx, n_add, Y, ldy, F, H, ldh);
    }
    GNN_LAUNCH_CHECK("add_rows_kernel");
    return GNN_OK;
}

extern "C" int32_t gnn_add_rows(const int32_t* rows, int32_t n_active, const void* X, int64_t ldx, void* Y, int64_t ldy, int32_t F,
                                int32_t dtype, void* stream_) {
    GNN_REQUIRE(n_active >= 0, GNN_ERR_INVALID_ARG, "negative size");
    return add_rows_impl(rows, n_active, X, ldx, n_active, Y, ldy, F, nullptr, 0, dtype, (hipStream_t)stream_);
}

extern "C" int32_t gnn_add_rows_masked(const int32_t* rows, int32_t n_active, const void* X, int64_t ldx, int32_t n_add, void* Y,
                                       int64_t ldy, int32_t F, const void* H, int64_t ldh, int32_t dtype, void* stream_) {
    GNN_REQUIRE(H != nullptr || n_active == 0 || F == 0, GNN_ERR_INVALID_ARG, "H is NULL");
    return add_rows_impl(rows, n_active, X, ldx, n_add, Y, ldy, F, H, ldh, dtype, (hipStream_t)stream_);
}
