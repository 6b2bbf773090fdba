// Source-blocked layout of the long rows of a plan.
//
// Section 4.2 of the paper blocks the SOURCE vertices: with one CSR per block of sources, a block of
// f_V stays in cache while every destination row sweeps over it, at the price of one pass over the
// output per block.  On this chip the caches that matter are the 4 MB L2s, and a pass over the
// output per block is affordable only for rows that have many edges per block.  So only the rows of
// at least `min_degree` edges take part: their neighbour lists, mapped to source RANKS (descending
// gather count) and sorted, are cut at the boundaries of rank blocks into pieces, and the pieces are
// laid out and processed block by block.  All rows that gather from a block do so within a short
// time, so a source row is fetched into an L2 once per block instead of once per gather; the pieces
// of a row write fp32 partial rows that a second kernel adds in a fixed order (deterministic, no
// atomics).  The short rows keep the plain path: they have too few edges per block, and their hot
// sources hit in the L2s anyway.
//
// Everything here is integer work, once per plan, and fully deterministic:
//   order of the edges:  (block of the source rank, row position in the plan, source rank)
//   pieces:              runs of equal (block, row), cut every `max_piece` edges
//   partial slot:        pieces of a row numbered in block order, rows back to back
#include <utility>

#include "common.h"

namespace {

// The piece kernel reads the per-edge streams four elements at a time and may run up to three
// elements past a piece's end: every stream is allocated with this many elements to spare.
constexpr int64_t kStreamPad = 8;

struct BlockMap {
    int32_t hot;         // block 0 = ranks [0, hot)
    int32_t block;       // blocks 1 .. n_blocks-2 hold `block` ranks each
    int32_t rest_begin;  // block n_blocks-1 = ranks [rest_begin, N)
    int32_t n_blocks;
};

__device__ __forceinline__ int block_of(const BlockMap m, int32_t r) {
    if (r < m.hot) return 0;
    if (r >= m.rest_begin) return m.n_blocks - 1;
    return 1 + (r - m.hot) / m.block;
}
__device__ __forceinline__ int32_t block_lo(const BlockMap m, int k) {
    if (k <= 0) return 0;
    if (k >= m.n_blocks) return INT32_MAX;
    if (k == m.n_blocks - 1) return m.rest_begin;
    const int64_t lo = int64_t(m.hot) + int64_t(k - 1) * m.block;
    return int32_t(lo < m.rest_begin ? lo : m.rest_begin);
}

int grid_for(int64_t n, int block, int64_t cap = (int64_t(1) << 16)) {
    int64_t g = (n + block - 1) / block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return static_cast<int>(g);
}

// h_of[i] = index (within the hot range) of the row that owns plan-order position p0 + i
__global__ void __launch_bounds__(256) blk_expand_rows_kernel(const int64_t *__restrict__ p_indptr, int64_t hot_begin,
                                                              int64_t n_hot, int64_t p0, uint32_t *__restrict__ h_of) {
    const int lane = threadIdx.x & 63;
    const int64_t n_waves = (int64_t(gridDim.x) * blockDim.x) >> 6;
    for (int64_t h = (int64_t(blockIdx.x) * blockDim.x + threadIdx.x) >> 6; h < n_hot; h += n_waves) {
        const int64_t b = p_indptr[hot_begin + h] - p0, e = p_indptr[hot_begin + h + 1] - p0;
        for (int64_t i = b + lane; i < e; i += 64) h_of[i] = uint32_t(h);
    }
}

__global__ void __launch_bounds__(256) blk_init_pairs_kernel(const int32_t *__restrict__ rank_indices, int64_t p0, int64_t n,
                                                             uint32_t *__restrict__ keys, uint32_t *__restrict__ vals) {
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride) {
        keys[i] = uint32_t(rank_indices[p0 + i]) & 0x7FFFFFFFu;  // bit 31 may carry a cold flag
        vals[i] = uint32_t(i);
    }
}

__global__ void __launch_bounds__(256) blk_gather_u32_kernel(const uint32_t *__restrict__ table, const uint32_t *__restrict__ idx,
                                                             int64_t n, uint32_t mask, uint32_t *__restrict__ out) {
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride) out[i] = table[idx[i]] & mask;
}

// first position in the sorted list r[0..n) whose rank is >= bound
__device__ __forceinline__ int64_t lower_bound_rank(const uint32_t *__restrict__ r, int64_t n, int32_t bound) {
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (int32_t(r[mid]) < bound) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// One thread per cell (block k, hot row h): where the row's sorted list enters block k, how many
// edges it has there, and how many pieces that makes.  Tables are [k][h].
__global__ void __launch_bounds__(256) blk_cells_kernel(const int64_t *__restrict__ p_indptr, int64_t hot_begin, int64_t n_hot,
                                                        int64_t p0, const uint32_t *__restrict__ sorted_r, BlockMap m,
                                                        int64_t max_piece, uint32_t *__restrict__ cell_start,
                                                        uint32_t *__restrict__ cell_count, uint32_t *__restrict__ cell_pieces) {
    const int64_t n_cells = int64_t(m.n_blocks) * n_hot;
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t c = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; c < n_cells; c += stride) {
        const int k = int(c / n_hot);
        const int64_t h = c - int64_t(k) * n_hot;
        const int64_t b = p_indptr[hot_begin + h] - p0, len = p_indptr[hot_begin + h + 1] - p0 - b;
        const int64_t s0 = lower_bound_rank(sorted_r + b, len, block_lo(m, k));
        const int64_t s1 = lower_bound_rank(sorted_r + b, len, block_lo(m, k + 1));
        cell_start[c] = uint32_t(s0);
        cell_count[c] = uint32_t(s1 - s0);
        cell_pieces[c] = uint32_t((s1 - s0 + max_piece - 1) / max_piece);
    }
}

// One thread per hot row: number of pieces of the row before each block (in place of the cell's
// piece count, which the caller has saved) and in total.
__global__ void __launch_bounds__(256) blk_row_prefix_kernel(int64_t n_hot, int n_blocks, const uint32_t *__restrict__ cell_pieces,
                                                             uint32_t *__restrict__ row_prefix, uint32_t *__restrict__ row_total) {
    const int64_t h = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (h >= n_hot) return;
    uint32_t run = 0;
    for (int k = 0; k < n_blocks; ++k) {
        const int64_t c = int64_t(k) * n_hot + h;
        row_prefix[c] = run;
        run += cell_pieces[c];
    }
    row_total[h] = run;
}

// One thread per cell: its piece descriptors (begin, length, partial slot, row index).
__global__ void __launch_bounds__(256) blk_fill_pieces_kernel(int64_t n_hot, int n_blocks, int64_t max_piece,
                                                              const uint32_t *__restrict__ cell_count,
                                                              const uint32_t *__restrict__ edge_off,
                                                              const uint32_t *__restrict__ piece_off,
                                                              const uint32_t *__restrict__ row_prefix,
                                                              const uint32_t *__restrict__ rowbase, int32_t *__restrict__ pieces,
                                                              uint16_t *__restrict__ piece_block) {
    const int64_t n_cells = int64_t(n_blocks) * n_hot;
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t c = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; c < n_cells; c += stride) {
        const int64_t cnt = cell_count[c];
        if (cnt == 0) continue;
        const int64_t h = c % n_hot;
        const uint32_t slot0 = rowbase[h] + row_prefix[c];
        int64_t j = 0;
        for (int64_t b = 0; b < cnt; b += max_piece, ++j) {
            int32_t *p = pieces + 4 * (int64_t(piece_off[c]) + j);
            p[0] = int32_t(edge_off[c] + uint32_t(b));
            p[1] = int32_t(cnt - b < max_piece ? cnt - b : max_piece);
            p[2] = int32_t(slot0 + uint32_t(j));
            p[3] = int32_t(h);
            if (piece_block) piece_block[int64_t(piece_off[c]) + j] = uint16_t(c / n_hot);
        }
    }
}

// One thread per edge of the row-major sorted lists: its place in the block-major order.
__global__ void __launch_bounds__(256) blk_scatter_edges_kernel(int64_t n, const uint32_t *__restrict__ h_of,
                                                                const uint32_t *__restrict__ sorted_r,
                                                                const uint32_t *__restrict__ sorted_pos,
                                                                const int64_t *__restrict__ p_indptr, int64_t hot_begin,
                                                                int64_t n_hot, int64_t p0, const int32_t *__restrict__ row_perm,
                                                                const void *__restrict__ indptr, int ip64, BlockMap m,
                                                                const uint32_t *__restrict__ cell_start,
                                                                const uint32_t *__restrict__ edge_off,
                                                                int32_t *__restrict__ blk_indices, uint32_t *__restrict__ blk_epos,
                                                                uint16_t *__restrict__ blk_idx16) {
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride) {
        const int64_t h = h_of[i];
        const int32_t r = int32_t(sorted_r[i]);
        const int k = block_of(m, r);
        const int64_t c = int64_t(k) * n_hot + h;
        const int64_t row_begin = p_indptr[hot_begin + h] - p0;
        const int64_t dest = int64_t(edge_off[c]) + (i - row_begin - int64_t(cell_start[c]));
        blk_indices[dest] = r;
        if (blk_idx16) blk_idx16[dest] = k < m.n_blocks - 1 ? uint16_t(r - block_lo(m, k)) : uint16_t(0);
        // CSR position of the edge: its offset within the row is the same in plan order and in the CSR
        const int64_t v = row_perm[hot_begin + h];
        const int64_t csr_begin = ip64 ? static_cast<const int64_t *>(indptr)[v] : int64_t(static_cast<const int32_t *>(indptr)[v]);
        blk_epos[dest] = uint32_t(csr_begin + (int64_t(sorted_pos[i]) - row_begin));
    }
}

template <typename T>
bool dev_alloc(T **p, int64_t n) { return hipMalloc(p, sizeof(T) * size_t(n > 0 ? n : 1)) == hipSuccess; }

}  // namespace

extern "C" GNN_API int gnn_plan_set_blocking(gnn_plan *plan, const gnn_blocking_params *params) {
    if (!plan) return GNN_ERR_INVALID_ARG;
    if (plan->blk_decided) return GNN_ERR_UNSUPPORTED;
    gnn_blocking_params p{};
    if (params) p = *params;
    if (p.hot_lines < 0 || p.block_lines < 0 || p.max_piece < 0 || p.rest_min_count < 0) return GNN_ERR_INVALID_ARG;
    if (p.hot_lines > INT32_MAX || p.block_lines > INT32_MAX || p.max_piece > 32767) return GNN_ERR_INVALID_ARG;
    // the threshold must be a boundary of the plan's count histogram: 0 .. 16, 18, 20, .. 32, 36, 40, .. 64, 72, ...
    if (p.rest_min_count > (1 << 20) ||
        gnn_count_bucket_lower_bound(gnn_count_bucket_of(p.rest_min_count)) != p.rest_min_count)
        return GNN_ERR_INVALID_ARG;
    if (p.min_degree > 0) {  // must be a boundary between two bins
        bool found = false;
        for (int i = 0; i < plan->params.n_thresholds; ++i) found |= plan->params.thresholds[i] == p.min_degree;
        if (!found) return GNN_ERR_INVALID_ARG;
    }
    plan->blocking = p;
    return GNN_OK;
}

extern "C" GNN_API int gnn_plan_blocked_sizes(const gnn_plan *plan, int64_t *n_rows, int64_t *n_edges, int64_t *n_pieces,
                                              int32_t *n_blocks) {
    if (!plan) return GNN_ERR_INVALID_ARG;
    const bool on = plan->blk_decided && plan->blk_n_pieces > 0;
    if (n_rows) *n_rows = on ? plan->blk_n_hot : 0;
    if (n_edges) *n_edges = on ? plan->blk_n_edges : 0;
    if (n_pieces) *n_pieces = on ? plan->blk_n_pieces : 0;
    if (n_blocks) *n_blocks = on ? plan->blk_n_blocks : 0;
    return GNN_OK;
}

extern "C" GNN_API int gnn_plan_export_blocked(const gnn_plan *plan, int32_t *indices, uint32_t *epos, int32_t *pieces,
                                               uint32_t *rowbase, int32_t *rank) {
    if (!plan) return GNN_ERR_INVALID_ARG;
    if (rank && plan->rank && plan->n_rows > 0)
        GNN_HIP_TRY(hipMemcpy(rank, plan->rank, sizeof(int32_t) * plan->n_rows, hipMemcpyDeviceToHost));
    if (!(plan->blk_decided && plan->blk_n_pieces > 0)) return GNN_OK;
    if (indices) GNN_HIP_TRY(hipMemcpy(indices, plan->blk_indices, sizeof(int32_t) * plan->blk_n_edges, hipMemcpyDeviceToHost));
    if (epos) GNN_HIP_TRY(hipMemcpy(epos, plan->blk_epos, sizeof(uint32_t) * plan->blk_n_edges, hipMemcpyDeviceToHost));
    if (pieces) GNN_HIP_TRY(hipMemcpy(pieces, plan->blk_pieces, sizeof(int32_t) * 4 * plan->blk_n_pieces, hipMemcpyDeviceToHost));
    if (rowbase) GNN_HIP_TRY(hipMemcpy(rowbase, plan->blk_rowbase, sizeof(uint32_t) * (plan->blk_n_hot + 1), hipMemcpyDeviceToHost));
    return GNN_OK;
}

int gnn_plan_blocked_partial(gnn_plan *plan, int slices, int line_floats) {
    if (!plan || slices < 1 || line_floats < 1) return GNN_ERR_INVALID_ARG;
    const int64_t need = plan->blk_n_pieces * int64_t(slices) * line_floats * int64_t(sizeof(float));
    if (need <= plan->blk_partial_bytes) return GNN_OK;
    (void)hipGetLastError();
    (void)hipFree(plan->blk_partial);
    plan->blk_partial = nullptr;
    plan->blk_partial_bytes = 0;
    if (hipMalloc(&plan->blk_partial, size_t(need)) != hipSuccess) return GNN_ERR_ALLOC;
    plan->blk_partial_bytes = need;
    return GNN_OK;
}

int gnn_plan_blocked_edge_scale(gnn_plan *plan, int mode, hipStream_t stream, const float **out) {
    if (!plan || !out || mode < 1 || mode > 3 || plan->blk_n_edges <= 0 || !plan->edge_scale[mode - 1]) return GNN_ERR_INVALID_ARG;
    float *&arr = plan->blk_edge_scale[mode - 1];
    if (!arr) {
        (void)hipGetLastError();
        if (hipMalloc(&arr, sizeof(float) * size_t(plan->blk_n_edges + kStreamPad)) != hipSuccess) { arr = nullptr; return GNN_ERR_ALLOC; }
        blk_gather_u32_kernel<<<grid_for(plan->blk_n_edges, 256), 256, 0, stream>>>(
            reinterpret_cast<const uint32_t *>(plan->edge_scale[mode - 1]), plan->blk_epos, plan->blk_n_edges, 0xFFFFFFFFu,
            reinterpret_cast<uint32_t *>(arr));
        if (hipGetLastError() != hipSuccess) {
            (void)hipFree(arr);
            arr = nullptr;
            return GNN_ERR_LAUNCH;
        }
    }
    *out = arr;
    return GNN_OK;
}

int gnn_plan_blocked_bound_weights(gnn_plan *plan, hipStream_t stream, const float **out) {
    if (!plan || !out || plan->blk_n_edges <= 0 || !plan->bound_w) return GNN_ERR_INVALID_ARG;
    if (!plan->blk_bound_w) {
        (void)hipGetLastError();
        if (hipMalloc(&plan->blk_bound_w, sizeof(float) * size_t(plan->blk_n_edges + kStreamPad)) != hipSuccess) {
            plan->blk_bound_w = nullptr;
            return GNN_ERR_ALLOC;
        }
        plan->bound_w_stale = true;
    }
    if (plan->bound_w_stale) {
        blk_gather_u32_kernel<<<grid_for(plan->blk_n_edges, 256), 256, 0, stream>>>(
            reinterpret_cast<const uint32_t *>(plan->bound_w), plan->blk_epos, plan->blk_n_edges, 0xFFFFFFFFu,
            reinterpret_cast<uint32_t *>(plan->blk_bound_w));
        if (hipGetLastError() != hipSuccess) return GNN_ERR_LAUNCH;
        plan->bound_w_stale = false;
    }
    *out = plan->blk_bound_w;
    return GNN_OK;
}

extern "C" GNN_API int gnn_plan_bind_edge_weights(gnn_plan *plan, const float *edge_w, void *stream) {
    if (!plan) return GNN_ERR_INVALID_ARG;
    plan->bound_w = edge_w;
    plan->bound_w_stale = true;
    if (edge_w && plan->blk_decided && plan->blk_n_pieces > 0) {
        const float *unused = nullptr;
        return gnn_plan_blocked_bound_weights(plan, static_cast<hipStream_t>(stream), &unused);
    }
    return GNN_OK;
}

int gnn_plan_blocked(gnn_plan *plan, const void *indptr, hipStream_t stream, gnn_blocked_layout *out) {
    *out = gnn_blocked_layout{};
    if (!plan) return GNN_ERR_INVALID_ARG;
    if (!plan->blk_decided) {
        if (!plan->rank_indices || !plan->p_indptr || !plan->rank || !indptr) return GNN_ERR_INVALID_ARG;
        const int64_t N = plan->n_rows, E = plan->n_edges;
        gnn_blocking_params prm = plan->blocking;
        const bool automatic = prm.min_degree == 0;
        // Defaults, from measurements on the 2.45 M-vertex and 233 K-vertex power-law graphs with the short rows
        // running beside the pieces (see the kernel profile): rows of >= 256 edges, block 0 = the 16,384
        // most-gathered sources, further blocks of 24,576 (three quarters of an L2: the short rows' lines pass
        // through the same L2s), pieces of at most 96 edges, and one last block for every source gathered fewer
        // than 16 times (their reuse is not worth a partial line per block and row).  Against 32,768 / 128 / 3:
        // F=100 5.28 -> 5.12 ms, F=256 9.99 -> 9.78, F=512 20.0 -> 19.6; 233 K vertices F=602 13.58 -> 13.46.
        if (prm.min_degree == 0) prm.min_degree = 256;
        if (prm.hot_lines == 0) prm.hot_lines = 16384;
        if (prm.block_lines == 0) prm.block_lines = 24576;
        if (prm.max_piece == 0) prm.max_piece = 96;
        if (prm.rest_min_count == 0) prm.rest_min_count = 16;
        int first_bin = -1;
        for (int i = 0; i < plan->params.n_thresholds; ++i)
            if (plan->params.thresholds[i] == prm.min_degree) first_bin = i + 1;
        bool enable = prm.min_degree > 0 && first_bin > 0 && E > 0 && E < int64_t(INT32_MAX) && N > 0;
        int64_t hot_begin = 0, n_hot = 0, p0 = 0, n_edges = 0;
        if (enable) {
            hot_begin = plan->bin_offsets[first_bin];
            n_hot = N - hot_begin;
            enable = n_hot > 0;
        }
        if (enable) {
            GNN_HIP_TRY(hipMemcpyAsync(&p0, plan->p_indptr + hot_begin, 8, hipMemcpyDeviceToHost, stream));
            GNN_HIP_TRY(hipStreamSynchronize(stream));
            n_edges = E - p0;
            enable = n_edges > 0;
        }
        // Automatic gate: the gathered table must dwarf an L2 (else the plain path hits anyway), and the
        // long rows must hold a good part of the edges (else there is little to win).
        // (233 K vertices x 490 edges: F=256 6.29 -> 5.48 ms, F=602 15.05 -> 13.63)
        if (enable && automatic) enable = N >= 4 * int64_t(32768) && n_edges * 4 >= E;
        BlockMap m{};
        if (enable) {
            // sources gathered fewer than rest_min_count times share the last block (the threshold is a bucket boundary)
            int64_t rest_begin = 0;
            for (int b = 255; b >= gnn_count_bucket_of(prm.rest_min_count) && b >= 0; --b) rest_begin += plan->bucket_vertices[b];
            m.hot = int32_t(prm.hot_lines < N ? prm.hot_lines : N);
            m.block = int32_t(prm.block_lines);
            m.rest_begin = int32_t(rest_begin > m.hot ? rest_begin : m.hot);
            const int64_t n_mid = (int64_t(m.rest_begin) - m.hot + m.block - 1) / m.block;
            enable = n_mid + 2 <= 1024 && (n_mid + 2) * n_hot < (int64_t(1) << 31);
            m.n_blocks = int32_t(n_mid + 2);
        }
        if (enable) {
            (void)hipGetLastError();
            const int64_t n_cells = int64_t(m.n_blocks) * n_hot;
            uint32_t *h_of = nullptr, *buf_k[2] = {nullptr, nullptr}, *buf_v[2] = {nullptr, nullptr}, *table = nullptr, *sums = nullptr;
            uint32_t *cell_start = nullptr, *cell_count = nullptr, *cell_pieces = nullptr, *edge_off = nullptr, *row_prefix = nullptr;
            uint32_t *rowbase = nullptr, *blk_epos = nullptr;
            int32_t *blk_indices = nullptr, *pieces = nullptr;
            uint16_t *blk_idx16 = nullptr;
            uint16_t *piece_block = nullptr;
            const bool narrow = m.hot <= 65536 && m.block <= 65536;
            auto cleanup_tmp = [&]() {
                (void)hipFree(h_of); (void)hipFree(buf_k[0]); (void)hipFree(buf_k[1]); (void)hipFree(buf_v[0]); (void)hipFree(buf_v[1]);
                (void)hipFree(table); (void)hipFree(sums); (void)hipFree(cell_start); (void)hipFree(cell_count);
                (void)hipFree(cell_pieces); (void)hipFree(edge_off); (void)hipFree(row_prefix);
            };
            auto fail = [&](int s) {
                (void)hipStreamSynchronize(stream);
                cleanup_tmp();
                (void)hipFree(rowbase); (void)hipFree(blk_epos); (void)hipFree(blk_indices); (void)hipFree(pieces);
                (void)hipFree(blk_idx16); (void)hipFree(piece_block);
                return s;
            };
            const int64_t scan_n = n_cells > n_hot + 1 ? n_cells : n_hot + 1;
            const int64_t sums_n = gnn_sort_sums_elems(n_edges) > gnn_scan_sums_elems(scan_n) ? gnn_sort_sums_elems(n_edges) : gnn_scan_sums_elems(scan_n);
            bool ok = dev_alloc(&h_of, n_edges) && dev_alloc(&buf_k[0], n_edges) && dev_alloc(&buf_k[1], n_edges) &&
                      dev_alloc(&buf_v[0], n_edges) && dev_alloc(&buf_v[1], n_edges) &&
                      dev_alloc(&table, gnn_sort_table_elems(n_edges)) && dev_alloc(&sums, sums_n) &&
                      dev_alloc(&cell_start, n_cells) && dev_alloc(&cell_count, n_cells) && dev_alloc(&cell_pieces, n_cells + 1) &&
                      dev_alloc(&edge_off, n_cells + 1) && dev_alloc(&row_prefix, n_cells) && dev_alloc(&rowbase, n_hot + 1) &&
                      dev_alloc(&blk_indices, n_edges + kStreamPad) && dev_alloc(&blk_epos, n_edges + kStreamPad);
            if (ok && narrow) ok = dev_alloc(&blk_idx16, n_edges + kStreamPad);
            if (!ok) return fail(GNN_ERR_ALLOC);

            blk_expand_rows_kernel<<<grid_for(n_hot * 64, 256), 256, 0, stream>>>(plan->p_indptr, hot_begin, n_hot, p0, h_of);
            // sort the edges of the long rows by (row, source rank): first by rank, then, stably, by row
            blk_init_pairs_kernel<<<grid_for(n_edges, 256), 256, 0, stream>>>(plan->rank_indices, p0, n_edges, buf_k[0], buf_v[0]);
            if (hipGetLastError() != hipSuccess) return fail(GNN_ERR_LAUNCH);
            int where = 0;
            int rc = gnn_radix_sort_pairs(nullptr, buf_k, buf_v, n_edges, gnn_ilog2_ceil(N > 1 ? N : 2), table, sums, stream, &where);
            if (rc != GNN_OK) return fail(rc);
            if (where != 0) { std::swap(buf_k[0], buf_k[1]); std::swap(buf_v[0], buf_v[1]); }
            blk_gather_u32_kernel<<<grid_for(n_edges, 256), 256, 0, stream>>>(h_of, buf_v[0], n_edges, 0xFFFFFFFFu, buf_k[0]);
            rc = gnn_radix_sort_pairs(nullptr, buf_k, buf_v, n_edges, gnn_ilog2_ceil(n_hot > 1 ? n_hot : 2), table, sums, stream, &where);
            if (rc != GNN_OK) return fail(rc);
            uint32_t *sorted_pos = buf_v[where];      // plan-order offset (from p0) of the edge at each sorted position
            uint32_t *sorted_r = buf_k[where ^ 1];    // its source rank
            blk_gather_u32_kernel<<<grid_for(n_edges, 256), 256, 0, stream>>>(
                reinterpret_cast<const uint32_t *>(plan->rank_indices + p0), sorted_pos, n_edges, 0x7FFFFFFFu, sorted_r);
            blk_cells_kernel<<<grid_for(n_cells, 256), 256, 0, stream>>>(plan->p_indptr, hot_begin, n_hot, p0, sorted_r, m,
                                                                        prm.max_piece, cell_start, cell_count, cell_pieces);
            blk_row_prefix_kernel<<<grid_for(n_hot, 256, INT32_MAX), 256, 0, stream>>>(n_hot, m.n_blocks, cell_pieces, row_prefix, rowbase);
            if (hipGetLastError() != hipSuccess) return fail(GNN_ERR_LAUNCH);
            // block-major offsets of the cells' edges and pieces; partial slots of the rows
            if ((hipMemcpyAsync(edge_off, cell_count, sizeof(uint32_t) * n_cells, hipMemcpyDeviceToDevice, stream)) != hipSuccess) return fail(GNN_ERR_LAUNCH);
            if ((rc = gnn_scan_exclusive_u32(edge_off, n_cells, sums, stream)) != GNN_OK) return fail(rc);
            uint32_t last_cell_pieces = 0, last_piece_off = 0, last_row = 0, last_rowbase = 0;
            if ((hipMemcpyAsync(&last_cell_pieces, cell_pieces + n_cells - 1, 4, hipMemcpyDeviceToHost, stream)) != hipSuccess) return fail(GNN_ERR_LAUNCH);
            if ((hipMemcpyAsync(&last_row, rowbase + n_hot - 1, 4, hipMemcpyDeviceToHost, stream)) != hipSuccess) return fail(GNN_ERR_LAUNCH);
            if ((rc = gnn_scan_exclusive_u32(cell_pieces, n_cells, sums, stream)) != GNN_OK) return fail(rc);
            if ((rc = gnn_scan_exclusive_u32(rowbase, n_hot, sums, stream)) != GNN_OK) return fail(rc);
            if ((hipMemcpyAsync(&last_piece_off, cell_pieces + n_cells - 1, 4, hipMemcpyDeviceToHost, stream)) != hipSuccess) return fail(GNN_ERR_LAUNCH);
            if ((hipMemcpyAsync(&last_rowbase, rowbase + n_hot - 1, 4, hipMemcpyDeviceToHost, stream)) != hipSuccess) return fail(GNN_ERR_LAUNCH);
            if (hipStreamSynchronize(stream) != hipSuccess) return fail(GNN_ERR_LAUNCH);
            const int64_t n_pieces = int64_t(last_piece_off) + last_cell_pieces;
            const uint32_t total_slots = last_rowbase + last_row;
            if (int64_t(total_slots) != n_pieces || n_pieces <= 0 || n_pieces >= int64_t(INT32_MAX)) return fail(GNN_ERR_LAUNCH);
            if ((hipMemcpyAsync(rowbase + n_hot, &total_slots, 4, hipMemcpyHostToDevice, stream)) != hipSuccess) return fail(GNN_ERR_LAUNCH);
            if (!dev_alloc(&pieces, 4 * n_pieces)) return fail(GNN_ERR_ALLOC);
            if (narrow && !dev_alloc(&piece_block, n_pieces)) return fail(GNN_ERR_ALLOC);
            blk_fill_pieces_kernel<<<grid_for(n_cells, 256), 256, 0, stream>>>(n_hot, m.n_blocks, prm.max_piece, cell_count, edge_off,
                                                                              cell_pieces, row_prefix, rowbase, pieces, piece_block);
            blk_scatter_edges_kernel<<<grid_for(n_edges, 256), 256, 0, stream>>>(n_edges, h_of, sorted_r, sorted_pos, plan->p_indptr,
                                                                                hot_begin, n_hot, p0, plan->row_perm, indptr,
                                                                                plan->indptr_is_64, m, cell_start, edge_off,
                                                                                blk_indices, blk_epos, blk_idx16);
            if (hipGetLastError() != hipSuccess) return fail(GNN_ERR_LAUNCH);
            if (hipStreamSynchronize(stream) != hipSuccess) return fail(GNN_ERR_LAUNCH);
            cleanup_tmp();
            plan->blk_first_bin = first_bin;
            plan->blk_hot_begin = hot_begin;
            plan->blk_n_hot = n_hot;
            plan->blk_n_edges = n_edges;
            plan->blk_n_pieces = n_pieces;
            plan->blk_n_blocks = m.n_blocks;
            plan->blk_indices = blk_indices;
            plan->blk_epos = blk_epos;
            plan->blk_idx16 = blk_idx16;
            plan->blk_piece_block = piece_block;
            plan->blk_hot_lines = m.hot;
            plan->blk_block_lines = m.block;
            plan->blk_pieces = pieces;
            plan->blk_rowbase = rowbase;
        }
        plan->blk_decided = 1;
    }
    if (plan->blk_n_pieces > 0) {
        out->active = true;
        out->automatic = plan->blocking.min_degree == 0;
        out->first_bin = plan->blk_first_bin;
        out->hot_begin = plan->blk_hot_begin;
        out->n_hot = plan->blk_n_hot;
        out->n_pieces = plan->blk_n_pieces;
        out->indices = plan->blk_indices;
        out->epos = plan->blk_epos;
        out->idx16 = plan->blk_idx16;
        out->piece_block = plan->blk_piece_block;
        out->n_blocks = plan->blk_n_blocks;
        out->hot_lines = plan->blk_hot_lines;
        out->block_lines = plan->blk_block_lines;
        out->pieces = plan->blk_pieces;
        out->rowbase = plan->blk_rowbase;
    }
    return GNN_OK;
}
