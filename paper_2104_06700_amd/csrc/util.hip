// Status strings and the streaming-copy kernel of known traffic (a measured ceiling for the
// bench, and the calibration of the profiler's byte counters).
#include "common.h"

namespace {

__global__ void __launch_bounds__(256) copy16_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int64_t n) {
    int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
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
        case GNN_ERR_SCRATCH_CAPACITY: return "hub partial sums exceed the fixed scratch array of the no-allocation entry point";
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
