// Node-classification loss on the target vertices (paper section 8.1: the task is node
// classification): mean softmax cross-entropy and its gradient with respect to the logits.
// One wavefront per target row; the per-workgroup loss sums are combined by a single
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

template <int DT>
__global__ __launch_bounds__(256) void softmax_ce_kernel(const int32_t* __restrict__ rows, int32_t n_active,
                                                         const void* __restrict__ Z, int64_t ldz, int32_t C,
                                                         const int32_t* __restrict__ labels, void* __restrict__ dZ, int64_t lddz,
                                                         float* __restrict__ part) {
    __shared__ float s_loss[4];
    const int lane = lane_id(), wave = (int)(threadIdx.x >> 6);
    const int64_t i = (int64_t)blockIdx.x * 4 + wave;
    float row_loss = 0.f;
    if (i < n_active) {
        const int64_t v = rows ? (int64_t)rows[i] : i;
        const int32_t y = labels[i];
        float m = -INFINITY;
        for (int c = lane; c < C; c += kWave) m = fmaxf(m, ld_logit<DT>(Z, v * ldz + c));
        m = wave_max(m);
        float s = 0.f;
        for (int c = lane; c < C; c += kWave) s += expf(ld_logit<DT>(Z, v * ldz + c) - m);
        s = wave_sum(s);
        const float zy = (y >= 0 && y < C) ? ld_logit<DT>(Z, v * ldz + y) : m;
        row_loss = -(zy - m - logf(s));
        if (dZ) {
            const float inv_n = 1.0f / (float)n_active;
            for (int c = lane; c < C; c += kWave) {
                const float p = expf(ld_logit<DT>(Z, v * ldz + c) - m) / s;
                const float gval = (p - (c == y ? 1.f : 0.f)) * inv_n;
                if (DT == GNN_F32) ((float*)dZ)[v * lddz + c] = gval;
                else ((uint16_t*)dZ)[v * lddz + c] = f32_to_bf16(gval);
            }
        }
    }
    if (lane == 0) s_loss[wave] = row_loss;
    __syncthreads();
    if (threadIdx.x == 0) part[blockIdx.x] = (s_loss[0] + s_loss[1]) + (s_loss[2] + s_loss[3]);
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
    const int32_t n_part = n_active > 0 ? (n_active + 3) / 4 : 1;
    WsCarver carve(ws);
    float* part = carve.take<float>((size_t)n_part);
    bool query;
    GNN_CHECK(ws_protocol(ws, ws_bytes, carve.used, &query));
    if (query) return GNN_OK;
    GNN_REQUIRE(loss != nullptr, GNN_ERR_INVALID_ARG, "loss is NULL");
    if (n_active > 0) {
        GNN_REQUIRE(Z != nullptr && labels != nullptr, GNN_ERR_INVALID_ARG, "Z or labels is NULL");
        if (dtype == GNN_F32)
            softmax_ce_kernel<GNN_F32><<<n_part, 256, 0, stream>>>(rows, n_active, Z, ldz, C, labels, dZ, lddz, part);
        else
            softmax_ce_kernel<GNN_BF16><<<n_part, 256, 0, stream>>>(rows, n_active, Z, ldz, C, labels, dZ, lddz, part);
        GNN_LAUNCH_CHECK("softmax_ce_kernel");
    }
    loss_reduce_kernel<<<1, 1024, 0, stream>>>(part, n_active > 0 ? n_part : 0, n_active, loss);
    GNN_LAUNCH_CHECK("loss_reduce_kernel");
    return GNN_OK;
}
