// Shared host/device helpers of the gnnhot HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <stdio.h>
#include <stdarg.h>
#include "../../include/gnnhot.h"

namespace gnnhot {

constexpr int kWave = 64;

// ---- host side: error text, argument checks, workspace carving -------------------------
void set_error(const char* fmt, ...);

#define GNN_REQUIRE(cond, st, ...)                \
    do {                                          \
        if (!(cond)) {                            \
            gnnhot::set_error(__VA_ARGS__);       \
            return (int32_t)(st);                 \
        }                                         \
    } while (0)

#define GNN_HIP(call)                                                                  \
    do {                                                                               \
        hipError_t e_ = (call);                                                        \
        if (e_ != hipSuccess) {                                                        \
            gnnhot::set_error("%s failed: %s", #call, hipGetErrorString(e_));          \
            return (int32_t)GNN_ERR_HIP;                                               \
        }                                                                              \
    } while (0)

#define GNN_LAUNCH_CHECK(name)                                                         \
    do {                                                                               \
        hipError_t e_ = hipGetLastError();                                             \
        if (e_ != hipSuccess) {                                                        \
            gnnhot::set_error("launch of %s failed: %s", name, hipGetErrorString(e_)); \
            return (int32_t)GNN_ERR_HIP;                                               \
        }                                                                              \
    } while (0)

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Bump allocator over the caller's workspace; with base == nullptr it only measures.
struct WsCarver {
    char* base;
    size_t used = 0;
    explicit WsCarver(void* p) : base((char*)p) {}
    template <typename T>
    T* take(size_t count) {
        size_t off = used;
        used = align_up(used + count * sizeof(T), 256);
        return base ? (T*)(base + off) : nullptr;
    }
};

// Common (ws, ws_bytes) protocol.  Returns 1 if the call was only a size query.
inline int32_t ws_protocol(void* ws, size_t* ws_bytes, size_t need, bool* query_only) {
    *query_only = false;
    GNN_REQUIRE(ws_bytes != nullptr, GNN_ERR_INVALID_ARG, "ws_bytes is NULL");
    if (ws == nullptr) {
        *ws_bytes = need;
        *query_only = true;
        return GNN_OK;
    }
    GNN_REQUIRE(((uintptr_t)ws & 255u) == 0, GNN_ERR_INVALID_ARG, "ws is not 256-byte aligned");
    GNN_REQUIRE(*ws_bytes >= need, GNN_ERR_WORKSPACE, "workspace too small: %zu < %zu bytes", *ws_bytes, need);
    return GNN_OK;
}

inline int32_t check_csr(const gnn_csr* g, const char* what) {
    GNN_REQUIRE(g != nullptr, GNN_ERR_INVALID_ARG, "%s is NULL", what);
    GNN_REQUIRE(g->n_rows >= 0 && g->n_cols >= 0 && g->nnz >= 0, GNN_ERR_INVALID_ARG, "%s has a negative size", what);
    GNN_REQUIRE(g->nnz < ((int64_t)1 << 31), GNN_ERR_UNSUPPORTED, "%s: nnz %lld does not fit int32", what, (long long)g->nnz);
    GNN_REQUIRE(g->row_ptr != nullptr, GNN_ERR_INVALID_ARG, "%s: row_ptr is NULL", what);
    GNN_REQUIRE(g->col_idx != nullptr || g->nnz == 0, GNN_ERR_INVALID_ARG, "%s: col_idx is NULL", what);
    return GNN_OK;
}

#define GNN_CHECK(expr)                   \
    do {                                  \
        int32_t st_ = (expr);             \
        if (st_ != GNN_OK) return st_;    \
    } while (0)

inline int grid_for(int64_t items, int per_block, int max_blocks = 1 << 20) {
    int64_t b = (items + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > max_blocks) b = max_blocks;
    return (int)b;
}

// ---- device side ------------------------------------------------------------------------
// bfloat16 <-> float: the upper 16 bits of the float; round to nearest, ties to even.
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// gfx950 converts in hardware (v_cvt_pk_bf16_f32: round to nearest even, NaN stays NaN).
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    const __bf16 h = (__bf16)f;
    return __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ float bf16lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Orders LDS traffic between the lanes of ONE wavefront (no cross-wave meaning).
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <typename T>
__global__ void fill_kernel(T* p, int64_t n, T value) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = value;
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }

}  // namespace gnnhot
