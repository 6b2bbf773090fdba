// Status strings and the bandwidth calibration kernels the bench prints next to
// each result (a streaming copy, and a row gather from a table whose size
// decides whether it is served by L2, by the Infinity Cache or by HBM).
#include "common.h"

namespace {

__global__ void __launch_bounds__(256) copy16_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int64_t n) {
    int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

__device__ __forceinline__ uint64_t mix(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Each group of (row_bytes/16) lanes copies one pseudo-randomly chosen table row to out.
__global__ void __launch_bounds__(256) gather_rows_kernel(const uint4 *__restrict__ table, int64_t n_rows_table,
                                                          int lanes_per_row, uint4 *__restrict__ out,
                                                          int64_t n_rows_out, uint64_t seed) {
    const int64_t t = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t n_threads = int64_t(gridDim.x) * blockDim.x;
    const int64_t total = n_rows_out * lanes_per_row;
    for (int64_t i = t; i < total; i += n_threads) {
        const int64_t r = i / lanes_per_row;
        const int l = int(i - r * lanes_per_row);
        const int64_t src_row = int64_t(mix(seed ^ uint64_t(r)) % uint64_t(n_rows_table));
        out[i] = table[src_row * lanes_per_row + l];
    }
}

}  // namespace

extern "C" GNN_API const char *gnn_status_string(int status) {
    switch (status) {
        case GNN_OK: return "ok";
        case GNN_ERR_INVALID_ARG: return "invalid argument";
        case GNN_ERR_UNSUPPORTED: return "unsupported request";
        case GNN_ERR_ALLOC: return "allocation failed";
        case GNN_ERR_LAUNCH: return "HIP runtime error";
        case GNN_ERR_INVALID_GRAPH: return "graph violates the CSR preconditions";
        default: return "unknown status";
    }
}

extern "C" GNN_API int gnn_calib_copy(const void *src, void *dst, int64_t n_bytes, void *stream) {
    if (!src || !dst || n_bytes < 0 || n_bytes % 16) return GNN_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(src) % 16 || reinterpret_cast<uintptr_t>(dst) % 16) return GNN_ERR_INVALID_ARG;
    if (n_bytes == 0) return GNN_OK;
    const int64_t n = n_bytes / 16;
    int64_t grid = (n + 255) / 256;
    if (grid > 256 * 32) grid = 256 * 32;
    copy16_kernel<<<static_cast<int>(grid), 256, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), n);
    GNN_HIP_TRY(hipGetLastError());
    return GNN_OK;
}

extern "C" GNN_API int gnn_calib_gather(const void *table, int64_t n_rows_table, int64_t row_bytes, void *out,
                                int64_t n_rows_out, uint64_t seed, void *stream) {
    if (!table || !out || n_rows_table <= 0 || n_rows_out < 0 || row_bytes <= 0 || row_bytes % 16) return GNN_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(table) % 16 || reinterpret_cast<uintptr_t>(out) % 16) return GNN_ERR_INVALID_ARG;
    if (n_rows_out == 0) return GNN_OK;
    const int lanes = int(row_bytes / 16);
    int64_t grid = (n_rows_out * lanes + 255) / 256;
    if (grid > 256 * 64) grid = 256 * 64;
    gather_rows_kernel<<<static_cast<int>(grid), 256, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<const uint4 *>(table), n_rows_table, lanes, static_cast<uint4 *>(out), n_rows_out, seed);
    GNN_HIP_TRY(hipGetLastError());
    return GNN_OK;
}
