// Library-wide pieces: version, per-thread error text, normalisation factors, bitmaps.
#include "common.h"

namespace gnnhot {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

// out[v] = 1/len (mean) or len^-1/2 (symmetric GCN), 0 for an empty row.
__global__ __launch_bounds__(256) void norm_scales_kernel(int norm, const int32_t* __restrict__ len,
                                                          const int32_t* __restrict__ row_ptr, int32_t n,
                                                          float* __restrict__ out) {
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += (int64_t)gridDim.x * blockDim.x) {
        int32_t d = len ? len[v] : row_ptr[v + 1] - row_ptr[v];
        float r = 0.f;
        if (d > 0) r = norm == GNN_NORM_MEAN ? 1.0f / (float)d : 1.0f / sqrtf((float)d);
        out[v] = r;
    }
}

__global__ __launch_bounds__(256) void set_bits_kernel(const int32_t* __restrict__ ids, int32_t n_ids, int32_t n,
                                                       uint32_t* __restrict__ bitmap) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_ids; i += (int64_t)gridDim.x * blockDim.x) {
        int32_t v = ids[i];
        if (v >= 0 && v < n) atomicOr(&bitmap[v >> 5], 1u << (v & 31));
    }
}

}  // namespace gnnhot

using namespace gnnhot;

extern "C" int32_t gnn_version(void) { return 100; }

extern "C" const char* gnn_last_error(void) { return g_err; }

extern "C" int32_t gnn_norm_scales(int32_t norm, const int32_t* len, const int32_t* row_ptr, int32_t n, float* out,
                                   void* stream) {
    GNN_REQUIRE(norm == GNN_NORM_MEAN || norm == GNN_NORM_SYM, GNN_ERR_INVALID_ARG, "unknown norm %d", norm);
    GNN_REQUIRE(n >= 0, GNN_ERR_INVALID_ARG, "n < 0");
    if (n == 0) return GNN_OK;
    GNN_REQUIRE(out != nullptr && (len != nullptr || row_ptr != nullptr), GNN_ERR_INVALID_ARG, "NULL argument");
    norm_scales_kernel<<<grid_for(n, 256, 4096), 256, 0, (hipStream_t)stream>>>(norm, len, row_ptr, n, out);
    GNN_LAUNCH_CHECK("norm_scales_kernel");
    return GNN_OK;
}

extern "C" int32_t gnn_make_bitmap(const int32_t* ids, int32_t n_ids, int32_t n, uint32_t* bitmap, void* stream) {
    GNN_REQUIRE(n >= 0 && n_ids >= 0, GNN_ERR_INVALID_ARG, "negative size");
    if (n == 0) return GNN_OK;
    GNN_REQUIRE(bitmap != nullptr && (ids != nullptr || n_ids == 0), GNN_ERR_INVALID_ARG, "NULL argument");
    int64_t nw = ((int64_t)n + 31) / 32;
    fill_kernel<uint32_t><<<grid_for(nw, 256, 2048), 256, 0, (hipStream_t)stream>>>(bitmap, nw, 0u);
    GNN_LAUNCH_CHECK("fill_kernel");
    if (n_ids > 0) {
        set_bits_kernel<<<grid_for(n_ids, 256, 2048), 256, 0, (hipStream_t)stream>>>(ids, n_ids, n, bitmap);
        GNN_LAUNCH_CHECK("set_bits_kernel");
    }
    return GNN_OK;
}
