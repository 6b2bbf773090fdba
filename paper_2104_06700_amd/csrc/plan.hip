// Degree-binning plan: the GPU-side replacement for dynamic scheduling over
// destination rows of very different length (Section 4.2, "Multithreading").
//
// Rows are grouped by row-length bin with a stable multi-way split (ascending
// row id inside a bin), rows of the last bin are cut into fixed-size pieces, and
// the per-vertex column counts (needed for MEAN backward and GCN_SYM scaling)
// are histogrammed.  Everything is integer work and fully deterministic.
#include <new>

#include "common.h"

namespace {

constexpr int kSplitThreads = 1024;  // rows per workgroup in the split kernels
constexpr int kSplitWaves = kSplitThreads / 64;

struct Thresholds {
    int32_t k;
    int64_t t[GNN_MAX_THRESHOLDS];
};

__device__ __forceinline__ int64_t load_ip(const void *indptr, int ip64, int64_t i) {
    return ip64 ? static_cast<const int64_t *>(indptr)[i]
                : static_cast<int64_t>(static_cast<const int32_t *>(indptr)[i]);
}

__device__ __forceinline__ int bin_of(int64_t deg, const Thresholds &thr) {
    int b = 0;
    for (int i = 0; i < thr.k; ++i) b += (thr.t[i] <= deg) ? 1 : 0;
    return b;
}

__global__ void __launch_bounds__(256) count_cols_kernel(const int32_t *__restrict__ indices, int64_t E,
                                                         int32_t *__restrict__ col_counts) {
    int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t e = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; e < E; e += stride)
        atomicAdd(&col_counts[indices[e]], 1);
}

// 256 buckets over the count axis: counts below 16 one bucket each, then 8 buckets per octave.
__device__ __forceinline__ int count_bucket(int c) {
    if (c < 16) return c;
    const int o = 31 - __clz(c);
    return 16 + (o - 4) * 8 + ((c >> (o - 3)) & 7);
}

__global__ void __launch_bounds__(256) count_buckets_kernel(const int32_t *__restrict__ col_counts, int64_t N,
                                                            unsigned long long *__restrict__ vertices,
                                                            unsigned long long *__restrict__ edges) {
    __shared__ unsigned long long sv[256], se[256];
    sv[threadIdx.x] = 0;
    se[threadIdx.x] = 0;
    __syncthreads();
    int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t v = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; v < N; v += stride) {
        const int c = col_counts[v];
        const int b = count_bucket(c);
        atomicAdd(&sv[b], 1ull);  // integer sums: the order of the additions does not matter
        atomicAdd(&se[b], static_cast<unsigned long long>(c));
    }
    __syncthreads();
    if (sv[threadIdx.x]) atomicAdd(&vertices[threadIdx.x], sv[threadIdx.x]);
    if (se[threadIdx.x]) atomicAdd(&edges[threadIdx.x], se[threadIdx.x]);
}

// edges[b] += edges of the rows of bin b
__global__ void __launch_bounds__(256) bin_edges_kernel(const void *__restrict__ indptr, int ip64, int64_t N, Thresholds thr,
                                                        unsigned long long *__restrict__ edges) {
    __shared__ unsigned long long se[GNN_MAX_BINS];
    if (threadIdx.x < GNN_MAX_BINS) se[threadIdx.x] = 0;
    __syncthreads();
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t v = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; v < N; v += stride) {
        const int64_t deg = load_ip(indptr, ip64, v + 1) - load_ip(indptr, ip64, v);
        if (deg > 0) atomicAdd(&se[bin_of(deg, thr)], static_cast<unsigned long long>(deg));  // integer sums: any order
    }
    __syncthreads();
    if (threadIdx.x < GNN_MAX_BINS && se[threadIdx.x]) atomicAdd(&edges[threadIdx.x], se[threadIdx.x]);
}

// block_counts[b * n_blocks + blk] = rows of bin b among rows [blk*1024, blk*1024+1024)
__global__ void __launch_bounds__(kSplitThreads) bin_count_kernel(const void *__restrict__ indptr, int ip64,
                                                                  int64_t N, Thresholds thr, int64_t n_blocks,
                                                                  int64_t *__restrict__ block_counts) {
    __shared__ int counts[GNN_MAX_BINS];
    if (threadIdx.x < GNN_MAX_BINS) counts[threadIdx.x] = 0;
    __syncthreads();
    int64_t v = int64_t(blockIdx.x) * kSplitThreads + threadIdx.x;
    if (v < N) {
        int64_t deg = load_ip(indptr, ip64, v + 1) - load_ip(indptr, ip64, v);
        atomicAdd(&counts[bin_of(deg, thr)], 1);  // integer count: order does not matter
    }
    __syncthreads();
    if (threadIdx.x <= thr.k) block_counts[int64_t(threadIdx.x) * n_blocks + blockIdx.x] = counts[threadIdx.x];
}

// In-place exclusive prefix sum of data[0..n) by ONE workgroup; data[n] receives the total.
__global__ void __launch_bounds__(1024) scan_exclusive_kernel(int64_t *__restrict__ data, int64_t n) {
    __shared__ int64_t part[1024];
    const int t = threadIdx.x;
    const int64_t chunk = (n + 1023) / 1024;
    const int64_t lo = chunk * t < n ? chunk * t : n;
    const int64_t hi = lo + chunk < n ? lo + chunk : n;
    int64_t s = 0;
    for (int64_t i = lo; i < hi; ++i) s += data[i];
    part[t] = s;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {  // Hillis-Steele inclusive scan of the partial sums
        int64_t add = t >= off ? part[t - off] : 0;
        __syncthreads();
        part[t] += add;
        __syncthreads();
    }
    int64_t run = part[t] - s;  // exclusive prefix of this thread's chunk
    for (int64_t i = lo; i < hi; ++i) {
        int64_t x = data[i];
        data[i] = run;
        run += x;
    }
    if (t == 1023) data[n] = part[1023];
}

// Stable placement: row v goes to block_prefix[bin][blk] + (#rows of the same bin before it in the block).
__global__ void __launch_bounds__(kSplitThreads) bin_scatter_kernel(const void *__restrict__ indptr, int ip64,
                                                                    int64_t N, Thresholds thr, int64_t n_blocks,
                                                                    const int64_t *__restrict__ block_prefix,
                                                                    int32_t *__restrict__ row_perm) {
    __shared__ int wave_tot[kSplitWaves][GNN_MAX_BINS];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    int64_t v = int64_t(blockIdx.x) * kSplitThreads + threadIdx.x;
    int bin = -1;
    if (v < N) {
        int64_t deg = load_ip(indptr, ip64, v + 1) - load_ip(indptr, ip64, v);
        bin = bin_of(deg, thr);
    }
    int rank_in_wave = 0;
    for (int b = 0; b <= thr.k; ++b) {
        unsigned long long m = __ballot(bin == b);
        if (bin == b) rank_in_wave = __popcll(m & ((1ull << lane) - 1ull));
        if (lane == 0) wave_tot[wave][b] = __popcll(m);
    }
    __syncthreads();
    if (bin >= 0) {
        int before = 0;
        for (int w = 0; w < wave; ++w) before += wave_tot[w][bin];
        int64_t pos = block_prefix[int64_t(bin) * n_blocks + blockIdx.x] + before + rank_in_wave;
        row_perm[pos] = static_cast<int32_t>(v);
    }
}

__global__ void __launch_bounds__(256) hub_count_kernel(const int32_t *__restrict__ hub_rows, int64_t n_hub,
                                                        const void *__restrict__ indptr, int ip64, int64_t chunk,
                                                        int64_t *__restrict__ counts) {
    int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= n_hub) return;
    int64_t v = hub_rows[i];
    int64_t deg = load_ip(indptr, ip64, v + 1) - load_ip(indptr, ip64, v);
    counts[i] = (deg + chunk - 1) / chunk;
}

__global__ void __launch_bounds__(256) hub_fill_kernel(const int32_t *__restrict__ hub_rows, int64_t n_hub,
                                                       const void *__restrict__ indptr, int ip64, int64_t chunk,
                                                       const int64_t *__restrict__ offsets,
                                                       int64_t *__restrict__ chunks) {
    int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= n_hub) return;
    int64_t v = hub_rows[i];
    int64_t b = load_ip(indptr, ip64, v);
    const int64_t end = load_ip(indptr, ip64, v + 1);
    int64_t c = offsets[i];
    for (; b < end; b += chunk, ++c) {
        chunks[3 * c + 0] = v;
        chunks[3 * c + 1] = b;
        chunks[3 * c + 2] = b + chunk < end ? b + chunk : end;
    }
}

__global__ void __launch_bounds__(256) edge_scale_kernel(const int32_t *__restrict__ indices, int64_t E,
                                                         const int32_t *__restrict__ col_counts, int mode,
                                                         float *__restrict__ out) {
    int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t e = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; e < E; e += stride) {
        int c = col_counts[indices[e]];
        float d = static_cast<float>(c > 1 ? c : 1);
        out[e] = mode == 3 ? 1.0f / static_cast<float>(c + 1) : (mode == 1 ? 1.0f / d : 1.0f / sqrtf(d));
    }
}

int grid_for(int64_t n, int block, int64_t cap = (int64_t(1) << 20)) {
    int64_t g = (n + block - 1) / block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return static_cast<int>(g);
}

}  // namespace

extern "C" GNN_API void gnn_plan_default_params(gnn_plan_params *p) {
    if (!p) return;
    *p = gnn_plan_params{};
    const int64_t t[] = {1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024, 2048, 4096};
    p->n_thresholds = static_cast<int32_t>(sizeof(t) / sizeof(t[0]));
    for (int i = 0; i < p->n_thresholds; ++i) p->thresholds[i] = t[i];
    p->hub_chunk = 1024;
}

int gnn_plan_edge_scale(gnn_plan *plan, const int32_t *indices, int mode, hipStream_t stream, const float **out) {
    if (!plan || !out || mode < 1 || mode > 3) return GNN_ERR_INVALID_ARG;
    float *&arr = plan->edge_scale[mode - 1];
    if (!arr && plan->n_edges > 0) {
        if (!indices) return GNN_ERR_INVALID_ARG;
        (void)hipGetLastError();
        if (hipMalloc(&arr, sizeof(float) * plan->n_edges) != hipSuccess) { arr = nullptr; return GNN_ERR_ALLOC; }
        edge_scale_kernel<<<grid_for(plan->n_edges, 256, 1 << 16), 256, 0, stream>>>(indices, plan->n_edges, plan->col_counts, mode, arr);
        if (hipGetLastError() != hipSuccess) {  // an unfilled array must not serve a later call
            (void)hipFree(arr);
            arr = nullptr;
            return GNN_ERR_LAUNCH;
        }
    }
    *out = arr;
    return GNN_OK;
}

__global__ void __launch_bounds__(256) edge_operand_kernel(const float *__restrict__ fE, int64_t lde,
                                                           const int64_t *__restrict__ edge_ids, int64_t E,
                                                           float *__restrict__ out) {
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t e = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; e < E; e += stride) {
        const int64_t id = edge_ids ? edge_ids[e] : e;
        __builtin_nontemporal_store(fE[id * lde], out + e);
    }
}

int gnn_plan_edge_operand(gnn_plan *plan, const float *fE, int64_t lde, const int64_t *edge_ids, hipStream_t stream,
                          const float **out) {
    if (!plan || !out || !fE || lde < 1) return GNN_ERR_INVALID_ARG;
    *out = nullptr;
    if (plan->n_edges == 0) return GNN_OK;
    (void)hipGetLastError();
    if (!plan->edge_operand && hipMalloc(&plan->edge_operand, sizeof(float) * plan->n_edges) != hipSuccess) {
        plan->edge_operand = nullptr;
        return GNN_ERR_ALLOC;
    }
    edge_operand_kernel<<<grid_for(plan->n_edges, 256, 1 << 16), 256, 0, stream>>>(fE, lde, edge_ids, plan->n_edges, plan->edge_operand);
    if (hipGetLastError() != hipSuccess) return GNN_ERR_LAUNCH;
    *out = plan->edge_operand;
    return GNN_OK;
}

__global__ void __launch_bounds__(256) flag_cold_kernel(const int32_t *__restrict__ indices, int64_t E,
                                                        const int32_t *__restrict__ counts, int threshold,
                                                        int32_t *__restrict__ out) {
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t e = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; e < E; e += stride) {
        const int32_t u = indices[e];
        out[e] = counts[u] < threshold ? int32_t(uint32_t(u) | 0x80000000u) : u;
    }
}

// smallest count that falls into bucket b of count_bucket()
static int64_t bucket_lower_bound(int b) {
    if (b < 16) return b;
    const int o = 4 + (b - 16) / 8, m = (b - 16) % 8;
    return int64_t(8 + m) << (o - 3);
}

// Cold hints.  With column slices an XCD's L2 holds one line each of 32,768 rows; rows that are
// gathered rarely pass through it without ever being hit again and only displace warmer rows.
// Measured on the 2.45 M-vertex power-law graph: fetching the sources outside the ~160 K
// most-gathered vertices (13-19 % of the gathers) with non-temporal loads takes 4-6 % off a call
// (F=256: 13.45 -> 12.8 ms, F=100: 6.82 -> 6.4 ms), while marking warmer sources, or any sources
// of a graph whose vertices nearly all fit that set (the 233 K- and 133 K-vertex graphs), costs
// time: the non-temporal path is slower per byte and forfeits hits.  Hence the gate: the graph has
// at least 8 x 163,840 vertices and the cold sources receive 5-30 % of the gathers.
int gnn_plan_cold_indices(gnn_plan *plan, const int32_t *indices, bool force, hipStream_t stream, const int32_t **out) {
    *out = nullptr;
    if (!plan || plan->n_edges <= 0) return GNN_OK;
    if (plan->cold_decided && plan->cold_forced != (force ? 1 : 0)) {  // built under the other rule: build again
        (void)hipFree(plan->cold_indices);
        plan->cold_indices = nullptr;
        plan->cold_decided = 0;
    }
    if (!plan->cold_decided) {
        const int64_t warm = force ? (plan->n_rows + 3) / 4 : int64_t(5) * 32768;
        bool enable = force;
        if (!force && plan->n_rows >= 8 * warm) {
            const double cold_share = 1.0 - gnn_plan_top_share(plan, warm);
            enable = cold_share >= 0.05 && cold_share <= 0.30;
        }
        if (enable) {
            // count threshold: lower bound of the bucket in which the `warm` most-gathered vertices end
            int64_t seen = 0, thr = 1;
            for (int b = 255; b >= 0; --b) {
                seen += plan->bucket_vertices[b];
                if (seen >= warm) { thr = bucket_lower_bound(b); break; }
            }
            if (thr < 1) thr = 1;
            if (!indices) return GNN_ERR_INVALID_ARG;
            (void)hipGetLastError();
            if (hipMalloc(&plan->cold_indices, sizeof(int32_t) * plan->n_edges) != hipSuccess) {
                plan->cold_indices = nullptr;
                return GNN_ERR_ALLOC;
            }
            plan->cold_threshold = int32_t(thr > INT32_MAX ? INT32_MAX : thr);
            flag_cold_kernel<<<grid_for(plan->n_edges, 256, 1 << 16), 256, 0, stream>>>(indices, plan->n_edges, plan->col_counts,
                                                                                       plan->cold_threshold, plan->cold_indices);
            if (hipGetLastError() != hipSuccess) {
                (void)hipFree(plan->cold_indices);
                plan->cold_indices = nullptr;
                return GNN_ERR_LAUNCH;
            }
        }
        plan->cold_decided = 1;
        plan->cold_forced = force ? 1 : 0;
    }
    *out = plan->cold_indices;
    return GNN_OK;
}

// lens[i] = length of the row at position i of row_perm
__global__ void __launch_bounds__(256) plan_order_lens_kernel(const int32_t *__restrict__ row_perm, int64_t N,
                                                              const void *__restrict__ indptr, int ip64,
                                                              int64_t *__restrict__ lens) {
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < N; i += stride) {
        const int64_t v = row_perm[i];
        lens[i] = load_ip(indptr, ip64, v + 1) - load_ip(indptr, ip64, v);
    }
}

// One wavefront per row: copies the row's edge list to its plan-order position, mapping every
// source id to its rank and flagging the cold ones (rank >= warm) in bit 31.
__global__ void __launch_bounds__(256) plan_order_fill_kernel(const int32_t *__restrict__ row_perm, int64_t N,
                                                              const void *__restrict__ indptr, int ip64,
                                                              const int64_t *__restrict__ p_indptr,
                                                              const int32_t *__restrict__ indices,
                                                              const int32_t *__restrict__ rank, int64_t warm,
                                                              int32_t *__restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int64_t n_waves = int64_t(gridDim.x) * (blockDim.x >> 6);
    for (int64_t i = int64_t(blockIdx.x) * (blockDim.x >> 6) + (threadIdx.x >> 6); i < N; i += n_waves) {
        const int64_t v = row_perm[i];
        const int64_t o0 = load_ip(indptr, ip64, v), len = load_ip(indptr, ip64, v + 1) - o0;
        const int64_t p0 = p_indptr[i];
        for (int64_t k = lane; k < len; k += 64) {
            const int32_t r = rank[indices[o0 + k]];
            out[p0 + k] = r >= warm ? int32_t(uint32_t(r) | 0x80000000u) : r;
        }
    }
}

// The hub pieces in plan-order coordinates: (row, begin, end, original minus plan-order position).
__global__ void __launch_bounds__(256) plan_order_chunks_kernel(int64_t n_hub, int64_t hub_begin,
                                                                const void *__restrict__ indptr, int ip64,
                                                                const int64_t *__restrict__ p_indptr,
                                                                const int64_t *__restrict__ offsets,
                                                                const int64_t *__restrict__ chunks,
                                                                int64_t *__restrict__ p_chunks) {
    const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= n_hub) return;
    for (int64_t c = offsets[i]; c < offsets[i + 1]; ++c) {
        const int64_t v = chunks[3 * c];
        const int64_t delta = load_ip(indptr, ip64, v) - p_indptr[hub_begin + i];
        p_chunks[4 * c + 0] = v;
        p_chunks[4 * c + 1] = chunks[3 * c + 1] - delta;
        p_chunks[4 * c + 2] = chunks[3 * c + 2] - delta;
        p_chunks[4 * c + 3] = delta;
    }
}

// Rank layout.  The padded copy of the gathered matrix is plan-owned, so its row order is free:
// rows are stored by descending column count.  The dense tail table then holds the tails of the
// most-gathered vertices in its first lines (8 rows per line at F = 100), the warm part of the
// main table is one contiguous range, and the cold rule is exact (rank >= warm).  The index copy
// that maps sources to ranks is laid out in plan order at the same time, because the rows that a
// workgroup processes side by side are neighbours in row_perm, not in the CSR: read from the
// caller's CSR, their edge lists are scattered ~200-byte pieces whose 128-byte lines are fetched
// more than once.  Measured on the 2.45 M-vertex graph: rank order F=100 6.21 -> 6.05 ms, F=256
// 12.6 -> 12.26 ms; plan order on top of it: see the kernel profile.  The cold gate is that of
// gnn_plan_cold_indices.
int gnn_plan_rank_indices(gnn_plan *plan, const void *indptr, const int32_t *indices, bool force_cold, hipStream_t stream,
                          gnn_rank_layout *out) {
    *out = gnn_rank_layout{};
    if (!plan || plan->n_edges <= 0 || plan->n_rows <= 0) return GNN_OK;
    if (plan->rank_indices && plan->rank_forced != (force_cold ? 1 : 0)) {  // flagged under the other rule: build again
        (void)hipFree(plan->rank_indices);
        (void)hipFree(plan->p_indptr);
        (void)hipFree(plan->p_chunks);
        plan->rank_indices = nullptr;
        plan->p_indptr = nullptr;
        plan->p_chunks = nullptr;
    }
    if (!plan->rank_indices) {
        if (!indices || !indptr) return GNN_ERR_INVALID_ARG;
        const int64_t N = plan->n_rows;
        (void)hipGetLastError();
        if (!plan->rank) {
            if (hipMalloc(&plan->rank, sizeof(int32_t) * N) != hipSuccess) { plan->rank = nullptr; return GNN_ERR_ALLOC; }
            int rc = gnn_rank_by_count(plan->col_counts, N, plan->rank, stream);
            if (rc != GNN_OK) { (void)hipFree(plan->rank); plan->rank = nullptr; return rc; }
        }
        // The indices of this copy are ranks, so the kernel finds the cold sources by comparing with
        // the warm-set size of the call; bit 31 is only set when the tests force it.
        const int64_t warm = force_cold ? (N + 3) / 4 : N;
        int64_t *p_indptr = nullptr, *p_chunks = nullptr;
        int32_t *idx = nullptr;
        auto fail = [&](int s) { (void)hipFree(p_indptr); (void)hipFree(p_chunks); (void)hipFree(idx); return s; };
        if (hipMalloc(&p_indptr, sizeof(int64_t) * (N + 1)) != hipSuccess) return fail(GNN_ERR_ALLOC);
        if (hipMalloc(&idx, sizeof(int32_t) * plan->n_edges) != hipSuccess) return fail(GNN_ERR_ALLOC);
        if (plan->n_chunks > 0 && hipMalloc(&p_chunks, sizeof(int64_t) * 4 * plan->n_chunks) != hipSuccess) return fail(GNN_ERR_ALLOC);
        plan_order_lens_kernel<<<grid_for(N, 256), 256, 0, stream>>>(plan->row_perm, N, indptr, plan->indptr_is_64, p_indptr);
        scan_exclusive_kernel<<<1, 1024, 0, stream>>>(p_indptr, N);
        plan_order_fill_kernel<<<grid_for(N * 64, 256, 1 << 16), 256, 0, stream>>>(plan->row_perm, N, indptr, plan->indptr_is_64,
                                                                                   p_indptr, indices, plan->rank, warm, idx);
        if (plan->n_chunks > 0) {
            const int64_t hub_begin = plan->bin_offsets[plan->n_bins - 1];
            plan_order_chunks_kernel<<<grid_for(plan->n_hub_rows, 256), 256, 0, stream>>>(
                plan->n_hub_rows, hub_begin, indptr, plan->indptr_is_64, p_indptr, plan->hub_chunk_offsets, plan->chunks, p_chunks);
        }
        if (hipGetLastError() != hipSuccess) return fail(GNN_ERR_LAUNCH);
        plan->p_indptr = p_indptr;
        plan->p_chunks = p_chunks;
        plan->rank_indices = idx;
        plan->rank_forced = force_cold ? 1 : 0;
    }
    out->rank = plan->rank;
    out->indices = plan->rank_indices;
    out->cold_pays = false;
    if (plan->n_rows >= 8 * int64_t(5) * 32768) {  // the gate of gnn_plan_cold_indices
        const double cold_share = 1.0 - gnn_plan_top_share(plan, int64_t(5) * 32768);
        out->cold_pays = cold_share >= 0.05 && cold_share <= 0.30;
    }
    out->p_indptr = plan->p_indptr;
    out->p_chunks = plan->p_chunks;
    return GNN_OK;
}

double gnn_plan_top_share(const gnn_plan *plan, int64_t K) {
    if (!plan || plan->n_edges <= 0 || K <= 0) return 0.0;
    double edges = 0.0;
    int64_t left = K;
    for (int b = 255; b >= 0 && left > 0; --b) {
        const int64_t nv = plan->bucket_vertices[b];
        if (nv <= 0) continue;
        if (nv <= left) {
            edges += static_cast<double>(plan->bucket_edges[b]);
            left -= nv;
        } else {
            edges += static_cast<double>(plan->bucket_edges[b]) * static_cast<double>(left) / static_cast<double>(nv);
            left = 0;
        }
    }
    return edges / static_cast<double>(plan->n_edges);
}

extern "C" GNN_API double gnn_plan_gather_share(const gnn_plan *plan, int64_t K) { return gnn_plan_top_share(plan, K); }

int gnn_plan_padded(gnn_plan *plan, int64_t bytes) {
    if (!plan || bytes < 0) return GNN_ERR_INVALID_ARG;
    if (bytes <= plan->padded_bytes) return GNN_OK;
    (void)hipGetLastError();
    (void)hipFree(plan->padded);
    plan->padded = nullptr;
    plan->padded_bytes = 0;
    if (hipMalloc(&plan->padded, bytes) != hipSuccess) return GNN_ERR_ALLOC;
    // padding columns are never written again; clear them once so that they hold finite values
    if (hipMemset(plan->padded, 0, bytes) != hipSuccess) return GNN_ERR_LAUNCH;
    plan->padded_bytes = bytes;
    return GNN_OK;
}

extern "C" GNN_API int gnn_plan_prepare(gnn_plan *plan, const int32_t *indices, int op, int backward, int64_t F,
                                        int dtype, void *stream) {
    if (!plan || F < 0 || op < GNN_SUM || op > GNN_SAGE_GCN) return GNN_ERR_INVALID_ARG;
    if (dtype != GNN_F32 && dtype != GNN_BF16) return GNN_ERR_INVALID_ARG;
    int rc = gnn_plan_reserve(plan, F);
    if (rc != GNN_OK) return rc;
    const int esz = dtype == GNN_BF16 ? 2 : 4;
    {   // the padded copy a hot call on a dense, line-aligned matrix (ld = F) would use, if any
        // (a weight-less GCN call is assumed: with explicit weights the rows carry no factor)
        const bool scaled_source = ((op == GNN_MEAN || op == GNN_SAGE_GCN) && backward) || op == GNN_GCN_SYM;
        const gnn_layout layout = gnn_choose_layout(plan, plan->n_rows, F, esz, F, true, 0, 0, /*allow_tail=*/true, scaled_source,
                                                    gnn_plan_blocks_expected(plan, esz));
        if (layout.padded_copy) {
            rc = gnn_plan_padded(plan, layout.bytes);
            if (rc != GNN_OK) return rc;
            gnn_rank_layout unused{};  // built from the row pointers the plan was created from
            rc = gnn_plan_rank_indices(plan, plan->indptr_seen, indices, false, static_cast<hipStream_t>(stream), &unused);
            if (rc != GNN_OK) return rc;
            if (layout.slice_major) {  // the long rows as source-blocked pieces, and their partial sums
                gnn_blocked_layout bl{};
                rc = gnn_plan_blocked(plan, plan->indptr_seen, static_cast<hipStream_t>(stream), &bl);
                if (rc != GNN_OK) return rc;
                if (bl.active) {
                    int slices = 1;
                    while (slices < 8 && slices * 2 <= layout.main_lines) slices *= 2;
                    rc = gnn_plan_blocked_partial(plan, slices, 128 / esz);
                    if (rc != GNN_OK) return rc;
                    if (plan->bound_w) {
                        const float *unused_w = nullptr;
                        rc = gnn_plan_blocked_bound_weights(plan, static_cast<hipStream_t>(stream), &unused_w);
                        if (rc != GNN_OK) return rc;
                    }
                }
            }
        } else if (layout.slices_wanted) {  // the flagged index copy of the cold hints, where they pay
            const int32_t *unused_idx = nullptr;
            rc = gnn_plan_cold_indices(plan, indices, false, static_cast<hipStream_t>(stream), &unused_idx);
            if (rc != GNN_OK) return rc;
        }
    }
    const float *unused = nullptr;
    const int mode = (op == GNN_MEAN && backward) ? 1 : (op == GNN_GCN_SYM ? 2 : ((op == GNN_SAGE_GCN && backward) ? 3 : 0));
    if (mode) {
        rc = gnn_plan_edge_scale(plan, indices, mode, static_cast<hipStream_t>(stream), &unused);
        // ... and in the order of the source-blocked pieces, for the calls that read it there
        if (rc == GNN_OK && plan->blk_decided && plan->blk_n_pieces > 0 && plan->n_edges > 0)
            rc = gnn_plan_blocked_edge_scale(plan, mode, static_cast<hipStream_t>(stream), &unused);
    }
    return rc;
}

extern "C" GNN_API void gnn_plan_destroy(gnn_plan *plan) {
    if (!plan) return;
    (void)hipFree(plan->edge_scale[0]);
    (void)hipFree(plan->edge_scale[1]);
    (void)hipFree(plan->edge_scale[2]);
    (void)hipFree(plan->padded);
    (void)hipFree(plan->cold_indices);
    (void)hipFree(plan->rank);
    (void)hipFree(plan->rank_indices);
    (void)hipFree(plan->p_indptr);
    (void)hipFree(plan->p_chunks);
    (void)hipFree(plan->edge_operand);
    (void)hipFree(plan->blk_indices);
    (void)hipFree(plan->blk_epos);
    (void)hipFree(plan->blk_idx16);
    (void)hipFree(plan->blk_piece_block);
    (void)hipFree(plan->blk_pieces);
    (void)hipFree(plan->blk_rowbase);
    (void)hipFree(plan->blk_partial);
    for (int i = 0; i < 3; ++i) (void)hipFree(plan->blk_edge_scale[i]);
    (void)hipFree(plan->blk_bound_w);
    (void)hipFree(plan->row_perm);
    (void)hipFree(plan->col_counts);
    (void)hipFree(plan->chunks);
    (void)hipFree(plan->hub_chunk_offsets);
    (void)hipFree(plan->scratch);
    delete plan;
}

extern "C" GNN_API int gnn_plan_create(const void *indptr, const int32_t *indices, int64_t N, int indptr_is_64,
                               const gnn_plan_params *params, void *stream_v, gnn_plan **out) {
    if (!out) return GNN_ERR_INVALID_ARG;
    *out = nullptr;
    if (N < 0 || N > INT32_MAX || (N > 0 && !indptr)) return GNN_ERR_INVALID_ARG;
    gnn_plan_params prm;
    if (params) prm = *params; else gnn_plan_default_params(&prm);
    if (prm.n_thresholds < 0 || prm.n_thresholds > GNN_MAX_THRESHOLDS || prm.hub_chunk < 0)
        return GNN_ERR_INVALID_ARG;
    for (int i = 0; i < prm.n_thresholds; ++i) {
        if (prm.thresholds[i] <= 0) return GNN_ERR_INVALID_ARG;
        if (i > 0 && prm.thresholds[i] <= prm.thresholds[i - 1]) return GNN_ERR_INVALID_ARG;
    }
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    (void)hipGetLastError();  // a stale error of an earlier, failed call must not be blamed on this one
    gnn_plan *plan = new (std::nothrow) gnn_plan();
    if (!plan) return GNN_ERR_ALLOC;
    plan->n_rows = N;
    plan->n_bins = prm.n_thresholds + 1;
    plan->indptr_is_64 = indptr_is_64 ? 1 : 0;
    plan->params = prm;
    plan->indptr_seen = indptr;
    const int nb = plan->n_bins;
    for (int b = 0; b <= nb; ++b) plan->bin_offsets[b] = 0;
    if (N == 0) { *out = plan; return GNN_OK; }

    int status = GNN_OK;
    int64_t *block_counts = nullptr;
    auto fail = [&](int s) { (void)hipFree(block_counts); gnn_plan_destroy(plan); return s; };

    // number of edges = indptr[N]
    int64_t E = 0;
    if (indptr_is_64) {
        if (hipMemcpyAsync(&E, static_cast<const int64_t *>(indptr) + N, 8, hipMemcpyDeviceToHost, stream) != hipSuccess) return fail(GNN_ERR_LAUNCH);
        if (hipStreamSynchronize(stream) != hipSuccess) return fail(GNN_ERR_LAUNCH);
    } else {
        int32_t e32 = 0;
        if (hipMemcpyAsync(&e32, static_cast<const int32_t *>(indptr) + N, 4, hipMemcpyDeviceToHost, stream) != hipSuccess) return fail(GNN_ERR_LAUNCH);
        if (hipStreamSynchronize(stream) != hipSuccess) return fail(GNN_ERR_LAUNCH);
        E = e32;
    }
    if (E < 0 || (E > 0 && !indices)) return fail(GNN_ERR_INVALID_ARG);
    plan->n_edges = E;

    Thresholds thr{};
    thr.k = prm.n_thresholds;
    for (int i = 0; i < thr.k; ++i) thr.t[i] = prm.thresholds[i];

    const int64_t n_blocks = (N + kSplitThreads - 1) / kSplitThreads;
    const int64_t n_counts = n_blocks * nb;
    if (hipMalloc(&plan->row_perm, sizeof(int32_t) * N) != hipSuccess) return fail(GNN_ERR_ALLOC);
    if (hipMalloc(&plan->col_counts, sizeof(int32_t) * N) != hipSuccess) return fail(GNN_ERR_ALLOC);
    if (hipMalloc(&block_counts, sizeof(int64_t) * (n_counts + 1)) != hipSuccess) return fail(GNN_ERR_ALLOC);

    // column counts.  The zero fill is a kernel-free memset outside any graph capture.
    if (hipMemsetAsync(plan->col_counts, 0, sizeof(int32_t) * N, stream) != hipSuccess) return fail(GNN_ERR_LAUNCH);
    if (E > 0) count_cols_kernel<<<grid_for(E, 256, 1 << 16), 256, 0, stream>>>(indices, E, plan->col_counts);
    {   // bucket histogram of the column counts (for gnn_plan_top_share)
        unsigned long long *buckets = nullptr;
        if (hipMalloc(&buckets, sizeof(unsigned long long) * 512) != hipSuccess) return fail(GNN_ERR_ALLOC);
        bool ok = hipMemsetAsync(buckets, 0, sizeof(unsigned long long) * 512, stream) == hipSuccess;
        if (ok) {
            count_buckets_kernel<<<grid_for(N, 256, 2048), 256, 0, stream>>>(plan->col_counts, N, buckets, buckets + 256);
            unsigned long long host[512];
            ok = hipMemcpyAsync(host, buckets, sizeof(host), hipMemcpyDeviceToHost, stream) == hipSuccess &&
                 hipStreamSynchronize(stream) == hipSuccess;
            for (int b = 0; ok && b < 256; ++b) {
                plan->bucket_vertices[b] = static_cast<int64_t>(host[b]);
                plan->bucket_edges[b] = static_cast<int64_t>(host[256 + b]);
            }
        }
        (void)hipFree(buckets);
        if (!ok) return fail(GNN_ERR_LAUNCH);
    }

    {   // edges per bin (host copy: which share of the edges the long rows hold decides the layout of a call)
        unsigned long long *bin_edges = nullptr;
        if (hipMalloc(&bin_edges, sizeof(unsigned long long) * GNN_MAX_BINS) != hipSuccess) return fail(GNN_ERR_ALLOC);
        bool ok = hipMemsetAsync(bin_edges, 0, sizeof(unsigned long long) * GNN_MAX_BINS, stream) == hipSuccess;
        if (ok) {
            bin_edges_kernel<<<grid_for(N, 256, 2048), 256, 0, stream>>>(indptr, plan->indptr_is_64, N, thr, bin_edges);
            unsigned long long host[GNN_MAX_BINS];
            ok = hipMemcpyAsync(host, bin_edges, sizeof(host), hipMemcpyDeviceToHost, stream) == hipSuccess &&
                 hipStreamSynchronize(stream) == hipSuccess;
            for (int b = 0; ok && b < GNN_MAX_BINS; ++b) plan->bin_edges[b] = static_cast<int64_t>(host[b]);
        }
        (void)hipFree(bin_edges);
        if (!ok) return fail(GNN_ERR_LAUNCH);
    }

    // stable multi-way split of the rows by bin
    bin_count_kernel<<<static_cast<int>(n_blocks), kSplitThreads, 0, stream>>>(indptr, plan->indptr_is_64, N, thr, n_blocks, block_counts);
    scan_exclusive_kernel<<<1, 1024, 0, stream>>>(block_counts, n_counts);
    bin_scatter_kernel<<<static_cast<int>(n_blocks), kSplitThreads, 0, stream>>>(indptr, plan->indptr_is_64, N, thr, n_blocks, block_counts, plan->row_perm);
    if (hipGetLastError() != hipSuccess) return fail(GNN_ERR_LAUNCH);
    for (int b = 0; b < nb; ++b) {
        if (hipMemcpyAsync(&plan->bin_offsets[b], block_counts + int64_t(b) * n_blocks, 8, hipMemcpyDeviceToHost, stream) != hipSuccess)
            return fail(GNN_ERR_LAUNCH);
    }
    if (hipStreamSynchronize(stream) != hipSuccess) return fail(GNN_ERR_LAUNCH);
    plan->bin_offsets[nb] = N;

    // hub rows -> pieces
    if (prm.hub_chunk > 0) {
        const int64_t hub_begin = plan->bin_offsets[nb - 1];
        const int64_t n_hub = N - hub_begin;
        plan->n_hub_rows = n_hub;
        if (n_hub > 0) {
            if (hipMalloc(&plan->hub_chunk_offsets, sizeof(int64_t) * (n_hub + 1)) != hipSuccess) return fail(GNN_ERR_ALLOC);
            const int32_t *hub_rows = plan->row_perm + hub_begin;
            hub_count_kernel<<<grid_for(n_hub, 256), 256, 0, stream>>>(hub_rows, n_hub, indptr, plan->indptr_is_64, prm.hub_chunk, plan->hub_chunk_offsets);
            scan_exclusive_kernel<<<1, 1024, 0, stream>>>(plan->hub_chunk_offsets, n_hub);
            if (hipMemcpyAsync(&plan->n_chunks, plan->hub_chunk_offsets + n_hub, 8, hipMemcpyDeviceToHost, stream) != hipSuccess) return fail(GNN_ERR_LAUNCH);
            if (hipStreamSynchronize(stream) != hipSuccess) return fail(GNN_ERR_LAUNCH);
            if (plan->n_chunks > 0) {
                if (hipMalloc(&plan->chunks, sizeof(int64_t) * 3 * plan->n_chunks) != hipSuccess) return fail(GNN_ERR_ALLOC);
                hub_fill_kernel<<<grid_for(n_hub, 256), 256, 0, stream>>>(hub_rows, n_hub, indptr, plan->indptr_is_64, prm.hub_chunk, plan->hub_chunk_offsets, plan->chunks);
            }
        }
    }
    if (hipGetLastError() != hipSuccess) return fail(GNN_ERR_LAUNCH);
    if (hipStreamSynchronize(stream) != hipSuccess) return fail(GNN_ERR_LAUNCH);
    (void)hipFree(block_counts);
    (void)status;
    *out = plan;
    return GNN_OK;
}

extern "C" GNN_API int gnn_plan_sizes(const gnn_plan *plan, int64_t *n_rows, int32_t *n_bins, int64_t *n_chunks) {
    if (!plan) return GNN_ERR_INVALID_ARG;
    if (n_rows) *n_rows = plan->n_rows;
    if (n_bins) *n_bins = plan->n_bins;
    if (n_chunks) *n_chunks = plan->n_chunks;
    return GNN_OK;
}

extern "C" GNN_API int gnn_plan_export(const gnn_plan *plan, int64_t *bin_offsets, int32_t *row_perm, int64_t *chunks,
                               int32_t *col_counts) {
    if (!plan) return GNN_ERR_INVALID_ARG;
    if (bin_offsets) for (int b = 0; b <= plan->n_bins; ++b) bin_offsets[b] = plan->bin_offsets[b];
    if (row_perm && plan->n_rows > 0)
        GNN_HIP_TRY(hipMemcpy(row_perm, plan->row_perm, sizeof(int32_t) * plan->n_rows, hipMemcpyDeviceToHost));
    if (col_counts && plan->n_rows > 0)
        GNN_HIP_TRY(hipMemcpy(col_counts, plan->col_counts, sizeof(int32_t) * plan->n_rows, hipMemcpyDeviceToHost));
    if (chunks && plan->n_chunks > 0)
        GNN_HIP_TRY(hipMemcpy(chunks, plan->chunks, sizeof(int64_t) * 3 * plan->n_chunks, hipMemcpyDeviceToHost));
    return GNN_OK;
}

extern "C" GNN_API int64_t gnn_plan_workspace_bytes(const gnn_plan *plan, int64_t F) {
    if (!plan || F < 0) return 0;
    return plan->n_chunks * gnn_partial_ld(F) * int64_t(sizeof(float));
}

extern "C" GNN_API int gnn_plan_reserve(gnn_plan *plan, int64_t F) {
    if (!plan || F < 0) return GNN_ERR_INVALID_ARG;
    const int64_t need = gnn_plan_workspace_bytes(plan, F);
    if (need <= plan->scratch_bytes) return GNN_OK;
    (void)hipGetLastError();
    (void)hipFree(plan->scratch);
    plan->scratch = nullptr;
    plan->scratch_bytes = 0;
    if (hipMalloc(&plan->scratch, need) != hipSuccess) return GNN_ERR_ALLOC;
    plan->scratch_bytes = need;
    return GNN_OK;
}
