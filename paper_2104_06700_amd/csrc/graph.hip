// Once-per-graph structure kernels: CSR row pointers from a sorted destination
// array, the transposed graph (CSR by source) the backward pass runs over, and a
// precondition checker.  Integer work only; every result is deterministic.
//
// The paper takes the CSR as given (Section 4.1) and builds extra CSRs as
// preprocessing (Section 4.2); the transposed graph is what the implied
// backward pass needs.
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

// ---------------------------------------------------------------- stable radix sort
// LSD radix sort of (key, value) pairs of 32-bit words, 8 bits per pass, stable.  One wavefront
// owns a tile of kSortTile consecutive pairs.  Per pass: (1) every tile counts its digits,
// (2) the [digit][tile] table is prefix-summed (digit-major, so equal digits of earlier tiles come
// first), (3) every tile walks its pairs in order, 64 at a time, and places each behind the
// equal-digit pairs that precede it (lanes with the same digit are found with eight ballots).
constexpr int kSortRounds = 64;
constexpr int kSortTile = 64 * kSortRounds;

__device__ __forceinline__ unsigned long long same_digit_lanes(unsigned digit, bool valid) {
    unsigned long long peers = __ballot(valid);
#pragma unroll
    for (int bit = 0; bit < 8; ++bit) {
        const bool one = (digit >> bit) & 1u;
        const unsigned long long b = __ballot(one);
        peers &= one ? b : ~b;
    }
    return peers;
}

__global__ void __launch_bounds__(64) sort_count_kernel(const uint32_t *__restrict__ keys, int64_t n, int shift,
                                                        int64_t n_tiles, uint32_t *__restrict__ table) {
    __shared__ uint32_t hist[256];
    const int lane = threadIdx.x;
    for (int d = lane; d < 256; d += 64) hist[d] = 0;
    __syncthreads();
    const int64_t tile0 = int64_t(blockIdx.x) * kSortTile;
    for (int r = 0; r < kSortRounds; ++r) {
        const int64_t i = tile0 + int64_t(r) * 64 + lane;
        const bool valid = i < n;
        const unsigned digit = valid ? (keys[i] >> shift) & 255u : 0u;
        const unsigned long long peers = same_digit_lanes(digit, valid);
        if (valid && (peers & ((1ull << lane) - 1ull)) == 0) hist[digit] += __popcll(peers);  // one leader per digit
        __syncthreads();
    }
    for (int d = lane; d < 256; d += 64) table[int64_t(d) * n_tiles + blockIdx.x] = hist[d];
}

__global__ void __launch_bounds__(64) sort_scatter_kernel(const uint32_t *__restrict__ keys_in,
                                                          const uint32_t *__restrict__ vals_in, int64_t n, int shift,
                                                          int64_t n_tiles, const uint32_t *__restrict__ table,
                                                          uint32_t *__restrict__ keys_out,
                                                          uint32_t *__restrict__ vals_out) {
    __shared__ uint32_t base[256];
    const int lane = threadIdx.x;
    for (int d = lane; d < 256; d += 64) base[d] = table[int64_t(d) * n_tiles + blockIdx.x];
    __syncthreads();
    const int64_t tile0 = int64_t(blockIdx.x) * kSortTile;
    for (int r = 0; r < kSortRounds; ++r) {
        const int64_t i = tile0 + int64_t(r) * 64 + lane;
        const bool valid = i < n;
        const uint32_t key = valid ? keys_in[i] : 0u;
        const unsigned digit = (key >> shift) & 255u;
        const unsigned long long peers = same_digit_lanes(digit, valid);
        const unsigned long long before = peers & ((1ull << lane) - 1ull);
        uint32_t pos = 0;
        if (valid) pos = base[digit] + __popcll(before);
        __syncthreads();
        if (valid) {
            keys_out[pos] = key;
            vals_out[pos] = vals_in[i];
            if (before == 0) base[digit] += __popcll(peers);
        }
        __syncthreads();
    }
}

// Exclusive prefix sum of a uint32 table in three steps (block sums, scan of the sums, local scans).
constexpr int kScanItems = 16;
constexpr int kScanChunk = 256 * kScanItems;

__global__ void __launch_bounds__(256) scan_block_sums_kernel(const uint32_t *__restrict__ data, int64_t n,
                                                              uint32_t *__restrict__ sums) {
    __shared__ uint32_t red[256];
    const int64_t lo = int64_t(blockIdx.x) * kScanChunk + int64_t(threadIdx.x) * kScanItems;
    uint32_t s = 0;
    for (int k = 0; k < kScanItems; ++k) if (lo + k < n) s += data[lo + k];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (int(threadIdx.x) < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) sums[blockIdx.x] = red[0];
}

__global__ void __launch_bounds__(1024) scan_sums_kernel(uint32_t *__restrict__ sums, int64_t n) {
    __shared__ uint32_t part[1024];
    const int t = threadIdx.x;
    const int64_t chunk = (n + 1023) / 1024;
    const int64_t lo = chunk * t < n ? chunk * t : n;
    const int64_t hi = lo + chunk < n ? lo + chunk : n;
    uint32_t s = 0;
    for (int64_t i = lo; i < hi; ++i) s += sums[i];
    part[t] = s;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
        uint32_t add = t >= off ? part[t - off] : 0;
        __syncthreads();
        part[t] += add;
        __syncthreads();
    }
    uint32_t run = part[t] - s;
    for (int64_t i = lo; i < hi; ++i) {
        uint32_t x = sums[i];
        sums[i] = run;
        run += x;
    }
}

__global__ void __launch_bounds__(256) scan_local_kernel(uint32_t *__restrict__ data, int64_t n,
                                                         const uint32_t *__restrict__ sums_scanned) {
    __shared__ uint32_t part[256];
    const int t = threadIdx.x;
    const int64_t lo = int64_t(blockIdx.x) * kScanChunk + int64_t(t) * kScanItems;
    uint32_t v[kScanItems];
    uint32_t s = 0;
    for (int k = 0; k < kScanItems; ++k) {
        v[k] = lo + k < n ? data[lo + k] : 0;
        s += v[k];
    }
    part[t] = s;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
        uint32_t add = t >= off ? part[t - off] : 0;
        __syncthreads();
        part[t] += add;
        __syncthreads();
    }
    uint32_t run = sums_scanned[blockIdx.x] + part[t] - s;
    for (int k = 0; k < kScanItems; ++k) {
        if (lo + k < n) data[lo + k] = run;
        run += v[k];
    }
}

// Sorts n pairs by the low `bits` bits of the key.  buf_k[0]/buf_v[0] hold the input and are
// overwritten; the result ends in buf_k[*out]/buf_v[*out].  `first_keys` (optional) replaces
// buf_k[0] as the read-only input of the first pass.
int radix_sort_pairs(const uint32_t *first_keys, uint32_t *buf_k[2], uint32_t *buf_v[2], int64_t n, int bits,
                     uint32_t *table, uint32_t *sums, hipStream_t stream, int *out) {
    const int64_t n_tiles = (n + kSortTile - 1) / kSortTile;
    const int64_t n_table = n_tiles * 256;
    const int64_t n_sums = (n_table + kScanChunk - 1) / kScanChunk;
    if (n_tiles > INT32_MAX || n_sums > INT32_MAX) return GNN_ERR_UNSUPPORTED;
    int cur = 0;
    for (int shift = 0; shift < bits; shift += 8) {
        const uint32_t *kin = (shift == 0 && first_keys) ? first_keys : buf_k[cur];
        sort_count_kernel<<<static_cast<unsigned>(n_tiles), 64, 0, stream>>>(kin, n, shift, n_tiles, table);
        scan_block_sums_kernel<<<static_cast<unsigned>(n_sums), 256, 0, stream>>>(table, n_table, sums);
        scan_sums_kernel<<<1, 1024, 0, stream>>>(sums, n_sums);
        scan_local_kernel<<<static_cast<unsigned>(n_sums), 256, 0, stream>>>(table, n_table, sums);
        sort_scatter_kernel<<<static_cast<unsigned>(n_tiles), 64, 0, stream>>>(kin, buf_v[cur], n, shift, n_tiles, table,
                                                                             buf_k[cur ^ 1], buf_v[cur ^ 1]);
        if (hipGetLastError() != hipSuccess) return GNN_ERR_LAUNCH;
        cur ^= 1;
    }
    *out = cur;
    return GNN_OK;
}

__global__ void __launch_bounds__(256) rank_keys_kernel(const int32_t *__restrict__ counts, int64_t N,
                                                        uint32_t *__restrict__ keys, uint32_t *__restrict__ ids) {
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t v = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; v < N; v += stride) {
        keys[v] = ~uint32_t(counts[v]);  // ascending keys = descending counts
        ids[v] = uint32_t(v);
    }
}

__global__ void __launch_bounds__(256) rank_scatter_kernel(const uint32_t *__restrict__ ids_sorted, int64_t N,
                                                           int32_t *__restrict__ rank) {
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < N; i += stride) rank[ids_sorted[i]] = int32_t(i);
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

int gnn_radix_sort_pairs(const uint32_t *first_keys, uint32_t *buf_k[2], uint32_t *buf_v[2], int64_t n, int bits,
                         uint32_t *table, uint32_t *sums, hipStream_t stream, int *out) {
    return radix_sort_pairs(first_keys, buf_k, buf_v, n, bits, table, sums, stream, out);
}
int64_t gnn_sort_table_elems(int64_t n) { return (n + kSortTile - 1) / kSortTile * 256; }
int64_t gnn_sort_sums_elems(int64_t n) { return (gnn_sort_table_elems(n) + kScanChunk - 1) / kScanChunk + 1; }
int64_t gnn_scan_sums_elems(int64_t n) { return (n + kScanChunk - 1) / kScanChunk + 1; }
int gnn_scan_exclusive_u32(uint32_t *data, int64_t n, uint32_t *sums, hipStream_t stream) {
    if (n <= 0) return GNN_OK;
    const int64_t n_sums = (n + kScanChunk - 1) / kScanChunk;
    if (n_sums > INT32_MAX) return GNN_ERR_UNSUPPORTED;
    scan_block_sums_kernel<<<static_cast<unsigned>(n_sums), 256, 0, stream>>>(data, n, sums);
    scan_sums_kernel<<<1, 1024, 0, stream>>>(sums, n_sums);
    scan_local_kernel<<<static_cast<unsigned>(n_sums), 256, 0, stream>>>(data, n, sums);
    return hipGetLastError() == hipSuccess ? GNN_OK : GNN_ERR_LAUNCH;
}

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

    int32_t *row_of = nullptr;
    uint32_t *buf_k[2] = {nullptr, nullptr}, *buf_v[2] = {nullptr, nullptr}, *table = nullptr, *sums = nullptr;
    auto cleanup = [&]() {
        (void)hipFree(row_of); (void)hipFree(buf_k[0]); (void)hipFree(buf_k[1]); (void)hipFree(buf_v[0]);
        (void)hipFree(buf_v[1]); (void)hipFree(table); (void)hipFree(sums);
    };
    auto fail = [&](int s) { (void)hipStreamSynchronize(stream); cleanup(); return s; };

    const int64_t n_tiles = (E + kSortTile - 1) / kSortTile;
    const int64_t n_table = n_tiles * 256;
    const int64_t n_sums = (n_table + kScanChunk - 1) / kScanChunk;
    if (hipMalloc(&row_of, sizeof(int32_t) * E) != hipSuccess) return fail(GNN_ERR_ALLOC);
    for (int i = 0; i < 2; ++i) {
        if (hipMalloc(&buf_k[i], sizeof(uint32_t) * E) != hipSuccess) return fail(GNN_ERR_ALLOC);
        if (hipMalloc(&buf_v[i], sizeof(uint32_t) * E) != hipSuccess) return fail(GNN_ERR_ALLOC);
    }
    if (hipMalloc(&table, sizeof(uint32_t) * n_table) != hipSuccess) return fail(GNN_ERR_ALLOC);
    if (hipMalloc(&sums, sizeof(uint32_t) * (n_sums + 1)) != hipSuccess) return fail(GNN_ERR_ALLOC);

    if (indptr_is_64)
        expand_rows_kernel<int64_t><<<grid_for(N * 64, 256), 256, 0, stream>>>(static_cast<const int64_t *>(indptr), N, row_of);
    else
        expand_rows_kernel<int32_t><<<grid_for(N * 64, 256), 256, 0, stream>>>(static_cast<const int32_t *>(indptr), N, row_of);
    iota_kernel<<<grid_for(E, 256), 256, 0, stream>>>(buf_v[0], E);
    if (hipGetLastError() != hipSuccess) return fail(GNN_ERR_LAUNCH);

    // Stable sort of (source id, CSR position) on the bits a vertex id can occupy.
    const int bits = gnn_ilog2_ceil(N > 1 ? N : 2);
    int where = 0;
    rc = radix_sort_pairs(reinterpret_cast<const uint32_t *>(indices), buf_k, buf_v, E, bits, table, sums, stream, &where);
    if (rc != GNN_OK) return fail(rc);
    const int32_t *keys_sorted = reinterpret_cast<const int32_t *>(buf_k[where]);
    const uint32_t *pos_sorted = buf_v[where];

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

// rank[v] = position of vertex v when the vertices are ordered by descending count (equal counts
// by ascending id: the sort is stable).  Temporary buffers are allocated and freed here; synchronous.
int gnn_rank_by_count(const int32_t *counts, int64_t N, int32_t *rank, hipStream_t stream) {
    if (N <= 0) return GNN_OK;
    if (!counts || !rank || N > INT32_MAX) return GNN_ERR_INVALID_ARG;
    (void)hipGetLastError();
    uint32_t *buf_k[2] = {nullptr, nullptr}, *buf_v[2] = {nullptr, nullptr}, *table = nullptr, *sums = nullptr;
    auto cleanup = [&]() {
        (void)hipFree(buf_k[0]); (void)hipFree(buf_k[1]); (void)hipFree(buf_v[0]); (void)hipFree(buf_v[1]);
        (void)hipFree(table); (void)hipFree(sums);
    };
    auto fail = [&](int s) { (void)hipStreamSynchronize(stream); cleanup(); return s; };
    const int64_t n_tiles = (N + kSortTile - 1) / kSortTile;
    const int64_t n_table = n_tiles * 256;
    const int64_t n_sums = (n_table + kScanChunk - 1) / kScanChunk;
    for (int i = 0; i < 2; ++i) {
        if (hipMalloc(&buf_k[i], sizeof(uint32_t) * N) != hipSuccess) return fail(GNN_ERR_ALLOC);
        if (hipMalloc(&buf_v[i], sizeof(uint32_t) * N) != hipSuccess) return fail(GNN_ERR_ALLOC);
    }
    if (hipMalloc(&table, sizeof(uint32_t) * n_table) != hipSuccess) return fail(GNN_ERR_ALLOC);
    if (hipMalloc(&sums, sizeof(uint32_t) * (n_sums + 1)) != hipSuccess) return fail(GNN_ERR_ALLOC);
    rank_keys_kernel<<<grid_for(N, 256), 256, 0, stream>>>(counts, N, buf_k[0], buf_v[0]);
    if (hipGetLastError() != hipSuccess) return fail(GNN_ERR_LAUNCH);
    int where = 0;
    int rc = radix_sort_pairs(nullptr, buf_k, buf_v, N, 32, table, sums, stream, &where);
    if (rc != GNN_OK) return fail(rc);
    rank_scatter_kernel<<<grid_for(N, 256), 256, 0, stream>>>(buf_v[where], N, rank);
    if (hipGetLastError() != hipSuccess) return fail(GNN_ERR_LAUNCH);
    if (hipStreamSynchronize(stream) != hipSuccess) return fail(GNN_ERR_LAUNCH);
    cleanup();
    return GNN_OK;
}
