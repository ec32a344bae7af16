// Node-classification loss on the target vertices (paper section 8.1: the task is node
// classification): mean softmax cross-entropy and its gradient with respect to the logits.
// A group of 8 to 64 lanes per target row; the per-workgroup loss sums are combined by a single
// workgroup in a fixed order, so the scalar is bit-reproducible.
#include "common.h"

namespace gnnhot {

template <int DT>
__device__ __forceinline__ float ld_logit(const void* Z, int64_t off) {
    if (DT == GNN_F32) return ((const float*)Z)[off];
    return bf16_to_f32(((const uint16_t*)Z)[off]);
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x = fmaxf(x, __shfl_xor(x, d, kWave));
    return x;
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, kWave);
    return x;
}

// LW lanes (8, 16, 32 or 64) own one row, 256 / LW rows per workgroup and sweep; with C <= LW every lane keeps its
// logit in a register (one read of the row).  Rows are dealt to the lane groups in a fixed pattern and every group
// adds up its rows in order, so the loss does not depend on timing.
template <int DT, int LW>
__global__ __launch_bounds__(256) void softmax_ce_kernel(const int32_t* __restrict__ rows, int32_t n_active,
                                                         const void* __restrict__ Z, int64_t ldz, int32_t C,
                                                         const int32_t* __restrict__ labels, void* __restrict__ dZ, int64_t lddz,
                                                         float* __restrict__ part) {
    constexpr int GPB = 256 / LW;
    __shared__ float s_loss[GPB];
    const int grp = (int)threadIdx.x / LW, sl = (int)threadIdx.x % LW;
    const float inv_n = 1.0f / (float)n_active;
    float loss_acc = 0.f;
    for (int64_t base = (int64_t)blockIdx.x * GPB; base < n_active; base += (int64_t)gridDim.x * GPB) {  // uniform over the workgroup
        const int64_t i = base + grp;
        const bool active = i < n_active;
        const int64_t v = active ? (rows ? (int64_t)rows[i] : i) : 0;
        const int32_t y = active ? labels[i] : -1;
        float row_loss;
        if (C <= LW) {
            const bool mine = active && sl < C;
            const float z = mine ? ld_logit<DT>(Z, v * ldz + sl) : -INFINITY;
            float m = z;
#pragma unroll
            for (int d = LW / 2; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, kWave));
            const float e = mine ? expf(z - m) : 0.f;
            float sum = e;
#pragma unroll
            for (int d = LW / 2; d >= 1; d >>= 1) sum += __shfl_xor(sum, d, kWave);
            const bool y_ok = y >= 0 && y < C;
            const float zy_l = __shfl(z, (int)(threadIdx.x & 63) - sl + (y_ok ? y : 0), kWave);
            const float zy = y_ok ? zy_l : m;
            row_loss = active ? -(zy - m - logf(sum)) : 0.f;
            if (dZ && mine) {
                const float gval = (e / sum - (sl == y ? 1.f : 0.f)) * inv_n;
                if (DT == GNN_F32) ((float*)dZ)[v * lddz + sl] = gval;
                else ((uint16_t*)dZ)[v * lddz + sl] = f32_to_bf16(gval);
            }
        } else {  // LW == 64 here: three sweeps over the row
            float m = -INFINITY;
            if (active)
                for (int c = sl; c < C; c += LW) m = fmaxf(m, ld_logit<DT>(Z, v * ldz + c));
            m = wave_max(m);
            float sum = 0.f;
            if (active)
                for (int c = sl; c < C; c += LW) sum += expf(ld_logit<DT>(Z, v * ldz + c) - m);
            sum = wave_sum(sum);
            const float zy = (active && y >= 0 && y < C) ? ld_logit<DT>(Z, v * ldz + y) : m;
            row_loss = active ? -(zy - m - logf(sum)) : 0.f;
            if (dZ && active) {
                for (int c = sl; c < C; c += LW) {
                    const float p = expf(ld_logit<DT>(Z, v * ldz + c) - m) / sum;
                    const float gval = (p - (c == y ? 1.f : 0.f)) * inv_n;
                    if (DT == GNN_F32) ((float*)dZ)[v * lddz + c] = gval;
                    else ((uint16_t*)dZ)[v * lddz + c] = f32_to_bf16(gval);
                }
            }
        }
        loss_acc += row_loss;
    }
    if (sl == 0) s_loss[grp] = loss_acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
        for (int k = 0; k < GPB; ++k) t += s_loss[k];
        part[blockIdx.x] = t;
    }
}

__global__ __launch_bounds__(1024) void loss_reduce_kernel(const float* __restrict__ part, int32_t n_part, int32_t n_active,
                                                           float* __restrict__ loss) {
    __shared__ float s[1024];
    float t = 0.f;
    for (int i = threadIdx.x; i < n_part; i += 1024) t += part[i];
    s[threadIdx.x] = t;
    __syncthreads();
    for (int d = 512; d >= 1; d >>= 1) {
        if ((int)threadIdx.x < d) s[threadIdx.x] += s[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = n_active > 0 ? s[0] / (float)n_active : 0.f;
}

}  // namespace gnnhot

using namespace gnnhot;

extern "C" int32_t gnn_softmax_ce(const int32_t* rows, int32_t n_active, const void* Z, int64_t ldz, int32_t C,
                                  const int32_t* labels, void* dZ, int64_t lddz, int32_t dtype, float* loss, void* ws,
                                  size_t* ws_bytes, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    GNN_REQUIRE(n_active >= 0, GNN_ERR_INVALID_ARG, "negative row count");
    GNN_REQUIRE(dtype == GNN_F32 || dtype == GNN_BF16, GNN_ERR_UNSUPPORTED, "unknown dtype %d", dtype);
    GNN_REQUIRE(C >= 1 && C <= 1024, GNN_ERR_UNSUPPORTED, "C = %d out of range [1, 1024]", C);
    GNN_REQUIRE(ldz >= C && (dZ == nullptr || lddz >= C), GNN_ERR_SHAPE, "leading dimension smaller than C");
    const int lw = C <= 8 ? 8 : (C <= 16 ? 16 : (C <= 32 ? 32 : 64));
    const int64_t want = n_active > 0 ? ((int64_t)n_active + 256 / lw - 1) / (256 / lw) : 1;
    const int32_t n_part = (int32_t)(want < 4096 ? want : 4096);
    WsCarver carve(ws);
    float* part = carve.take<float>((size_t)n_part);
    bool query;
    GNN_CHECK(ws_protocol(ws, ws_bytes, carve.used, &query));
    if (query) return GNN_OK;
    GNN_REQUIRE(loss != nullptr, GNN_ERR_INVALID_ARG, "loss is NULL");
    if (n_active > 0) {
        GNN_REQUIRE(Z != nullptr && labels != nullptr, GNN_ERR_INVALID_ARG, "Z or labels is NULL");
#define GNN_CE(DT_, LW_) softmax_ce_kernel<DT_, LW_><<<n_part, 256, 0, stream>>>(rows, n_active, Z, ldz, C, labels, dZ, lddz, part)
        if (dtype == GNN_F32) {
            if (lw == 8) GNN_CE(GNN_F32, 8);
            else if (lw == 16) GNN_CE(GNN_F32, 16);
            else if (lw == 32) GNN_CE(GNN_F32, 32);
            else GNN_CE(GNN_F32, 64);
        } else {
            if (lw == 8) GNN_CE(GNN_BF16, 8);
            else if (lw == 16) GNN_CE(GNN_BF16, 16);
            else if (lw == 32) GNN_CE(GNN_BF16, 32);
            else GNN_CE(GNN_BF16, 64);
        }
#undef GNN_CE
        GNN_LAUNCH_CHECK("softmax_ce_kernel");
    }
    loss_reduce_kernel<<<1, 1024, 0, stream>>>(part, n_active > 0 ? n_part : 0, n_active, loss);
    GNN_LAUNCH_CHECK("loss_reduce_kernel");
    return GNN_OK;
}
