// Once-per-graph structure kernels: CSR row pointers from a sorted destination
// array, the transposed graph (CSR by source) the backward pass runs over, and a
// precondition checker.  Integer work only; every result is deterministic.
//
// The paper takes the CSR as given (Section 4.1) and builds extra CSRs as
// preprocessing (Section 4.2); the transposed graph is what the implied
// backward pass needs.
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>

#include "common.h"

namespace {

template <typename IP>
__global__ void __launch_bounds__(256) indptr_from_sorted_kernel(const int32_t *__restrict__ keys, int64_t E,
                                                                 int64_t N, IP *__restrict__ indptr) {
    // Thread e (0..E) owns the boundary between keys[e-1] and keys[e]; it writes
    // indptr[v] = e for every v in (keys[e-1], keys[e]].  Each indptr entry has one writer.
    int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t e = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; e <= E; e += stride) {
        int64_t prev = e == 0 ? -1 : keys[e - 1];
        int64_t cur = e == E ? N : keys[e];
        for (int64_t v = prev + 1; v <= cur; ++v) indptr[v] = static_cast<IP>(e);
    }
}

// row_of[e] = v for e in [indptr[v], indptr[v+1]) -- one wavefront per row.
template <typename IP>
__global__ void __launch_bounds__(256) expand_rows_kernel(const IP *__restrict__ indptr, int64_t N,
                                                          int32_t *__restrict__ row_of) {
    const int lane = threadIdx.x & 63;
    int64_t wave = (int64_t(blockIdx.x) * blockDim.x + threadIdx.x) >> 6;
    int64_t n_waves = (int64_t(gridDim.x) * blockDim.x) >> 6;
    for (int64_t v = wave; v < N; v += n_waves) {
        int64_t b = indptr[v], e = indptr[v + 1];
        for (int64_t i = b + lane; i < e; i += 64) row_of[i] = static_cast<int32_t>(v);
    }
}

__global__ void __launch_bounds__(256) iota_kernel(uint32_t *__restrict__ out, int64_t n) {
    int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride)
        out[i] = static_cast<uint32_t>(i);
}

__global__ void __launch_bounds__(256) gather_transposed_kernel(const uint32_t *__restrict__ pos_sorted, int64_t E,
                                                                const int32_t *__restrict__ row_of,
                                                                const float *__restrict__ w,
                                                                int32_t *__restrict__ indices_t,
                                                                int64_t *__restrict__ perm, float *__restrict__ wt) {
    int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < E; i += stride) {
        uint32_t p = pos_sorted[i];
        indices_t[i] = row_of[p];
        if (perm) perm[i] = static_cast<int64_t>(p);
        if (wt) wt[i] = w[p];
    }
}

template <typename IP>
__global__ void __launch_bounds__(256) validate_kernel(const IP *__restrict__ indptr, const int32_t *__restrict__ indices,
                                                       int64_t N, int64_t E, int *__restrict__ bad) {
    int64_t stride = int64_t(gridDim.x) * blockDim.x;
    int64_t t0 = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    int err = 0;
    for (int64_t v = t0; v < N; v += stride)
        if (indptr[v] > indptr[v + 1]) err = 1;
    if (t0 == 0 && (indptr[0] != 0 || static_cast<int64_t>(indptr[N]) != E)) err = 1;
    for (int64_t e = t0; e < E; e += stride)
        if (indices[e] < 0 || indices[e] >= N) err = 1;
    if (err) atomicOr(bad, 1);
}

int grid_for(int64_t n, int block, int64_t cap = (int64_t(1) << 16)) {
    int64_t g = (n + block - 1) / block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return static_cast<int>(g);
}

int read_edge_count(const void *indptr, int64_t N, int ip64, hipStream_t stream, int64_t *E) {
    if (ip64) {
        GNN_HIP_TRY(hipMemcpyAsync(E, static_cast<const int64_t *>(indptr) + N, 8, hipMemcpyDeviceToHost, stream));
        GNN_HIP_TRY(hipStreamSynchronize(stream));
    } else {
        int32_t e32 = 0;
        GNN_HIP_TRY(hipMemcpyAsync(&e32, static_cast<const int32_t *>(indptr) + N, 4, hipMemcpyDeviceToHost, stream));
        GNN_HIP_TRY(hipStreamSynchronize(stream));
        *E = e32;
    }
    return GNN_OK;
}

}  // namespace

extern "C" GNN_API int gnn_csr_from_sorted_coo(const int32_t *dst_sorted, int64_t E, int64_t N, void *indptr_out,
                                       int indptr_is_64, void *stream_v) {
    if (N < 0 || E < 0 || !indptr_out || (E > 0 && !dst_sorted)) return GNN_ERR_INVALID_ARG;
    if (!indptr_is_64 && E > INT32_MAX) return GNN_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    (void)hipGetLastError();  // a stale error of an earlier, failed call must not be blamed on this one
    if (indptr_is_64)
        indptr_from_sorted_kernel<int64_t><<<grid_for(E + 1, 256), 256, 0, stream>>>(dst_sorted, E, N, static_cast<int64_t *>(indptr_out));
    else
        indptr_from_sorted_kernel<int32_t><<<grid_for(E + 1, 256), 256, 0, stream>>>(dst_sorted, E, N, static_cast<int32_t *>(indptr_out));
    GNN_HIP_TRY(hipGetLastError());
    return GNN_OK;
}

extern "C" GNN_API int gnn_transpose_csr(const void *indptr, const int32_t *indices, const float *edge_w, int64_t N,
                                 int indptr_is_64, void *indptr_t, int32_t *indices_t, int64_t *perm,
                                 float *edge_w_t, void *stream_v) {
    if (N < 0 || N > INT32_MAX || !indptr || !indptr_t) return GNN_ERR_INVALID_ARG;
    if (edge_w && !edge_w_t) return GNN_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    (void)hipGetLastError();
    int64_t E = 0;
    int rc = read_edge_count(indptr, N, indptr_is_64, stream, &E);
    if (rc != GNN_OK) return rc;
    if (E < 0 || E > int64_t(UINT32_MAX)) return GNN_ERR_INVALID_ARG;
    if (E > 0 && (!indices || !indices_t)) return GNN_ERR_INVALID_ARG;
    if (E == 0) {
        GNN_HIP_TRY(hipMemsetAsync(indptr_t, 0, (indptr_is_64 ? 8 : 4) * (N + 1), stream));
        GNN_HIP_TRY(hipStreamSynchronize(stream));
        return GNN_OK;
    }

    int32_t *row_of = nullptr, *keys_sorted = nullptr;
    uint32_t *pos = nullptr, *pos_sorted = nullptr;
    void *temp = nullptr;
    size_t temp_bytes = 0;
    auto cleanup = [&]() {
        (void)hipFree(row_of); (void)hipFree(keys_sorted); (void)hipFree(pos); (void)hipFree(pos_sorted); (void)hipFree(temp);
    };
    auto fail = [&](int s) { (void)hipStreamSynchronize(stream); cleanup(); return s; };

    if (hipMalloc(&row_of, sizeof(int32_t) * E) != hipSuccess) return fail(GNN_ERR_ALLOC);
    if (hipMalloc(&keys_sorted, sizeof(int32_t) * E) != hipSuccess) return fail(GNN_ERR_ALLOC);
    if (hipMalloc(&pos, sizeof(uint32_t) * E) != hipSuccess) return fail(GNN_ERR_ALLOC);
    if (hipMalloc(&pos_sorted, sizeof(uint32_t) * E) != hipSuccess) return fail(GNN_ERR_ALLOC);

    if (indptr_is_64)
        expand_rows_kernel<int64_t><<<grid_for(N * 64, 256), 256, 0, stream>>>(static_cast<const int64_t *>(indptr), N, row_of);
    else
        expand_rows_kernel<int32_t><<<grid_for(N * 64, 256), 256, 0, stream>>>(static_cast<const int32_t *>(indptr), N, row_of);
    iota_kernel<<<grid_for(E, 256), 256, 0, stream>>>(pos, E);
    if (hipGetLastError() != hipSuccess) return fail(GNN_ERR_LAUNCH);

    // Stable LSD radix sort of (source id, CSR position) on the bits a vertex id can occupy.
    const unsigned end_bit = static_cast<unsigned>(gnn_ilog2_ceil(N > 1 ? N : 2));
    const uint32_t *keys_in = reinterpret_cast<const uint32_t *>(indices);
    uint32_t *keys_out = reinterpret_cast<uint32_t *>(keys_sorted);
    if (rocprim::radix_sort_pairs(nullptr, temp_bytes, keys_in, keys_out, pos, pos_sorted, static_cast<size_t>(E), 0u,
                                  end_bit, stream) != hipSuccess)
        return fail(GNN_ERR_LAUNCH);
    if (hipMalloc(&temp, temp_bytes > 0 ? temp_bytes : 16) != hipSuccess) return fail(GNN_ERR_ALLOC);
    if (rocprim::radix_sort_pairs(temp, temp_bytes, keys_in, keys_out, pos, pos_sorted, static_cast<size_t>(E), 0u,
                                  end_bit, stream) != hipSuccess)
        return fail(GNN_ERR_LAUNCH);

    rc = gnn_csr_from_sorted_coo(keys_sorted, E, N, indptr_t, indptr_is_64, stream);
    if (rc != GNN_OK) return fail(rc);
    gather_transposed_kernel<<<grid_for(E, 256), 256, 0, stream>>>(pos_sorted, E, row_of, edge_w, indices_t, perm,
                                                                   edge_w ? edge_w_t : nullptr);
    if (hipGetLastError() != hipSuccess) return fail(GNN_ERR_LAUNCH);
    if (hipStreamSynchronize(stream) != hipSuccess) return fail(GNN_ERR_LAUNCH);
    cleanup();
    return GNN_OK;
}

extern "C" GNN_API int gnn_validate_csr(const void *indptr, const int32_t *indices, int64_t N, int64_t E, int indptr_is_64,
                                void *stream_v) {
    if (N < 0 || E < 0 || !indptr || (E > 0 && !indices)) return GNN_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    (void)hipGetLastError();
    int *bad = nullptr;
    if (hipMalloc(&bad, sizeof(int)) != hipSuccess) return GNN_ERR_ALLOC;
    int host_bad = 0;
    int rc = GNN_OK;
    if (hipMemsetAsync(bad, 0, sizeof(int), stream) != hipSuccess) rc = GNN_ERR_LAUNCH;
    if (rc == GNN_OK) {
        int64_t work = (N > E ? N : E) + 1;
        if (indptr_is_64)
            validate_kernel<int64_t><<<grid_for(work, 256), 256, 0, stream>>>(static_cast<const int64_t *>(indptr), indices, N, E, bad);
        else
            validate_kernel<int32_t><<<grid_for(work, 256), 256, 0, stream>>>(static_cast<const int32_t *>(indptr), indices, N, E, bad);
        if (hipGetLastError() != hipSuccess) rc = GNN_ERR_LAUNCH;
    }
    if (rc == GNN_OK && hipMemcpyAsync(&host_bad, bad, sizeof(int), hipMemcpyDeviceToHost, stream) != hipSuccess) rc = GNN_ERR_LAUNCH;
    if (rc == GNN_OK && hipStreamSynchronize(stream) != hipSuccess) rc = GNN_ERR_LAUNCH;
    (void)hipFree(bad);
    if (rc != GNN_OK) return rc;
    return host_bad ? GNN_ERR_INVALID_GRAPH : GNN_OK;
}
