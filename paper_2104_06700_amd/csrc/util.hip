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

// Bare gather of 128-byte lines: 8 lanes fetch one line with 16-byte loads, 16 lines in flight per lane group,
// the sums go nowhere but one float per thread.  What the memory system delivers when nothing else is asked of
// the kernel: the ceiling the gather kernels are held against.
__global__ void __launch_bounds__(256) line_gather_probe_kernel(const float *__restrict__ table, uint32_t last_line,
                                                                const uint32_t *__restrict__ ids, int64_t ids_per_group,
                                                                float *__restrict__ out) {
    constexpr int U = 16;
    const int lane = threadIdx.x & 63;
    const int sub = lane & 7;
    const int64_t thread = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    const uint32_t *my = ids + (thread >> 3) * ids_per_group;
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int64_t e = 0; e + U <= ids_per_group; e += U) {
        uint32_t s[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            s[u] = my[e + u];
            if (s[u] > last_line) s[u] = last_line;  // stays inside the table whatever the ids hold
        }
        float4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = *reinterpret_cast<const float4 *>(table + int64_t(s[u]) * 32 + sub * 4);
#pragma unroll
        for (int u = 0; u < U; ++u) { acc[0] += v[u].x; acc[1] += v[u].y; acc[2] += v[u].z; acc[3] += v[u].w; }
    }
    out[thread] = acc[0] + acc[1] + acc[2] + acc[3];
}

extern "C" GNN_API int gnn_calib_gather(const void *table, int64_t n_lines, const uint32_t *line_ids, int64_t n_ids, float *out,
                                        int64_t out_elems, void *stream) {
    if (!table || !line_ids || !out || n_lines <= 0 || n_lines > (int64_t(1) << 31) || n_ids < 0) return GNN_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(table) % 128) return GNN_ERR_INVALID_ARG;
    const int64_t blocks = 32768, groups = blocks * 256 / 8;
    const int64_t per = n_ids / groups / 16 * 16;
    if (per < 16 || out_elems < blocks * 256) return GNN_ERR_INVALID_ARG;
    line_gather_probe_kernel<<<static_cast<int>(blocks), 256, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<const float *>(table), uint32_t(n_lines - 1), line_ids, per, out);
    GNN_HIP_TRY(hipGetLastError());
    return GNN_OK;
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
