// Internal declarations shared by the translation units of libgnnagg.so.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gnnagg.h"

#define GNN_HIP_TRY(expr)                                  \
    do {                                                   \
        hipError_t gnn_err_ = (expr);                      \
        if (gnn_err_ != hipSuccess) return GNN_ERR_LAUNCH; \
    } while (0)

#define GNN_MAX_BINS (GNN_MAX_THRESHOLDS + 1)

// One plan = one graph orientation.  All pointers are device memory owned by
// the plan unless marked host.
struct gnn_plan {
    int64_t n_rows = 0;
    int64_t n_edges = 0;
    int32_t n_bins = 0;
    int32_t indptr_is_64 = 0;
    gnn_plan_params params{};
    int64_t bin_offsets[GNN_MAX_BINS + 1] = {0};  // host copy
    int64_t bin_edges[GNN_MAX_BINS] = {0};        // edges of the rows of each bin (host)
    int32_t *row_perm = nullptr;      // [n_rows]
    int32_t *col_counts = nullptr;    // [n_rows] occurrences of each vertex in indices
    // hub rows = rows of the last bin when params.hub_chunk > 0
    int64_t n_hub_rows = 0;
    int64_t n_chunks = 0;
    int64_t *chunks = nullptr;        // [n_chunks * 3] (row, e_begin, e_end)
    int64_t *hub_chunk_offsets = nullptr;  // [n_hub_rows + 1] first piece of each hub row
    // plan-owned scratch for hub partial sums
    void *scratch = nullptr;
    int64_t scratch_bytes = 0;
    const void *indptr_seen = nullptr;  // the indptr the plan was built from (sanity check only)
    // per-edge factor of the gathered vertex, streamed by the hot kernels:
    // [0] 1/max(c,1)   [1] 1/sqrt(max(c,1))   [2] 1/(c+1), c = col_counts[indices[e]]; built on first use
    float *edge_scale[3] = {nullptr, nullptr, nullptr};
    // Histogram of the column counts in 256 roughly logarithmic buckets (host copies): how many
    // vertices fall in each bucket and how many edges they are gathered by.  It answers "which
    // share of the gathers goes to the K most-gathered vertices", the quantity that decides
    // whether XCD column slices can keep more useful rows in L2.
    int64_t bucket_vertices[256] = {0};
    int64_t bucket_edges[256] = {0};
    // copy of the gathered matrix with rows padded to whole 128-byte lines (grown on first use)
    void *padded = nullptr;
    int64_t padded_bytes = 0;
    // copy of `indices` in which bit 31 marks the rarely gathered ("cold") sources; built on first
    // use when the plan's graph is in the regime where non-temporal loads of cold rows pay
    int32_t *cold_indices = nullptr;
    int32_t cold_decided = 0;    // 0: not yet; 1: decided (cold_indices is null when it does not pay)
    int32_t cold_threshold = 0;  // sources gathered fewer times than this are cold
    int32_t cold_forced = 0;     // the copy was built under GNN_FLAG_FORCE_COLD_HINTS (a call without it rebuilds)
    int32_t rank_forced = 0;     // likewise for rank_indices
    // Rank layout of the padded copy: rank[v] = position of v by descending column count; the copy
    // stores row v at row rank[v] and the kernels gather through rank_indices[e] =
    // rank[indices[e]] (bit 31: cold).  Built on first use.
    int32_t *rank = nullptr;
    int32_t *rank_indices = nullptr;
    // ... and in PLAN ORDER: the edge list of the row at position i of row_perm occupies
    // rank_indices[p_indptr[i] .. p_indptr[i+1]), so the rows a workgroup processes side by side read
    // one contiguous stretch of the index stream.  p_chunks: the hub pieces in those coordinates,
    // (row, begin, end, original position minus plan-order position) each.
    int64_t *p_indptr = nullptr;
    int64_t *p_chunks = nullptr;
    // a caller's scalar edge operand brought into CSR order (gnn_plan_edge_operand); refilled per call
    float *edge_operand = nullptr;
    // Source-blocked layout of the long rows (see gnn_plan_blocked); built on first use.
    gnn_blocking_params blocking{};   // requested parameters (zeros: automatic)
    int32_t blk_decided = 0;          // 0: not yet; 1: decided (blk_n_pieces == 0 when it does not apply)
    int32_t blk_first_bin = 0;        // rows of bins >= this are processed as pieces
    int64_t blk_hot_begin = 0;        // their range in row_perm is [blk_hot_begin, n_rows)
    int64_t blk_n_hot = 0;
    int64_t blk_n_edges = 0;          // edges of those rows
    int64_t blk_n_pieces = 0;
    int32_t blk_n_blocks = 0;
    int32_t *blk_indices = nullptr;   // [blk_n_edges] source ranks, block-major piece order
    uint32_t *blk_epos = nullptr;     // [blk_n_edges] CSR position of each (the caller's per-edge streams are read there)
    // blk_indices again as 16-bit offsets from the first rank of each edge's block, for the kernel to
    // read in place of the 32-bit ranks in all blocks but the last (whose range is not bounded); null
    // when a block spans more than 65,536 ranks.  blk_piece_block[p] = block of piece p.
    uint16_t *blk_idx16 = nullptr;
    uint16_t *blk_piece_block = nullptr;
    int32_t blk_hot_lines = 0, blk_block_lines = 0;
    int32_t *blk_pieces = nullptr;    // [blk_n_pieces * 4] (begin, length, partial slot, row index in the hot range)
    uint32_t *blk_rowbase = nullptr;  // [blk_n_hot + 1] first partial slot of each hot row
    float *blk_edge_scale[3] = {nullptr, nullptr, nullptr};  // edge_scale[m] at blk_epos, i.e. in the order of blk_indices
    // Edge weights the caller declared static (gnn_plan_bind_edge_weights): the pointer they were bound
    // under and their copy in the order of blk_indices, which the pieces of calls that pass that pointer
    // stream instead of reading the caller's array at blk_epos.
    const float *bound_w = nullptr;
    float *blk_bound_w = nullptr;
    bool bound_w_stale = false;       // the copy is older than the last binding
    void *blk_partial = nullptr;      // fp32 partial sums of one launch: [slices][blk_n_pieces][floats per line]
    int64_t blk_partial_bytes = 0;
};

// Source blocking (the GPU reading of Section 4.2's blocks of source vertices, applied to the long
// rows only).  Rows of at least `min_degree` edges are cut into pieces along blocks of source RANK
// (block 0 = the `hot_lines` most-gathered sources, then blocks of `block_lines`, then one block for
// the sources gathered fewer than `rest_min_count` times), and the pieces are processed block by
// block: all rows that gather from a block do so within a short time, so a source row is fetched
// into an L2 once per block instead of once per gather.  Pieces write fp32 partial rows that a
// second kernel adds in a fixed order.
struct gnn_blocked_layout {
    bool active;
    bool automatic;          // the plan chose to block by itself (no gnn_plan_set_blocking with a degree)
    int32_t first_bin;       // bins >= this are served by pieces
    int64_t hot_begin, n_hot, n_pieces;
    const int32_t *indices;  // block-major
    const uint32_t *epos;
    // 16-bit form of `indices` (null: none): piece p lies in block k = piece_block[p], which begins at
    // rank 0 (k = 0) or hot_lines + (k - 1) * block_lines; the last block keeps the 32-bit ranks
    const uint16_t *idx16;
    const uint16_t *piece_block;
    int32_t n_blocks, hot_lines, block_lines;
    const int32_t *pieces;
    const uint32_t *rowbase;
};
// Builds the layout on first use (allocation; needs the rank layout) and reports it.  Inactive when
// the graph or the plan's thresholds do not suit it.
int gnn_plan_blocked(gnn_plan *plan, const void *indptr, hipStream_t stream, gnn_blocked_layout *out);
// Makes plan->blk_partial large enough for `slices` column slices of `line_floats` floats per piece.
int gnn_plan_blocked_partial(gnn_plan *plan, int slices, int line_floats);
// The plan's per-edge factor stream `mode` (gnn_plan_edge_scale, which must have been built) in the order
// of the block-major index array; built on first use (allocation).
int gnn_plan_blocked_edge_scale(gnn_plan *plan, int mode, hipStream_t stream, const float **out);
// The bound edge weights in piece order: refreshed on `stream` when a binding is newer than the copy
// (allocates on first use).  Needs the layout and a binding.
int gnn_plan_blocked_bound_weights(gnn_plan *plan, hipStream_t stream, const float **out);

// Stable LSD radix sort of 32-bit (key, value) pairs on the low `bits` bits (graph.hip).  buf_k[0] /
// buf_v[0] hold the input (first_keys, if given, replaces buf_k[0] as read-only input of the first
// pass); the result is in buf_k[*out] / buf_v[*out].  table / sums: scratch of gnn_sort_table_elems(n)
// and gnn_sort_sums_elems(n) words.
int gnn_radix_sort_pairs(const uint32_t *first_keys, uint32_t *buf_k[2], uint32_t *buf_v[2], int64_t n, int bits,
                         uint32_t *table, uint32_t *sums, hipStream_t stream, int *out);
int64_t gnn_sort_table_elems(int64_t n);
int64_t gnn_sort_sums_elems(int64_t n);
// In-place exclusive prefix sum of n 32-bit words; sums: scratch of gnn_scan_sums_elems(n) words.
int gnn_scan_exclusive_u32(uint32_t *data, int64_t n, uint32_t *sums, hipStream_t stream);
int64_t gnn_scan_sums_elems(int64_t n);

// The 256 buckets over the count axis that a plan's histogram uses (plan.hip: count_bucket): counts below 16 one
// bucket each, then 8 buckets per octave.  Host-side twins for code that turns a count threshold into a rank.
static inline int gnn_count_bucket_of(int64_t c) {
    if (c < 16) return c < 0 ? 0 : int(c);
    int o = 0;
    while ((c >> (o + 1)) > 0) ++o;
    const int b = 16 + (o - 4) * 8 + int((c >> (o - 3)) & 7);
    return b > 255 ? 255 : b;
}
static inline int64_t gnn_count_bucket_lower_bound(int b) {
    if (b < 16) return b;
    const int o = 4 + (b - 16) / 8, m = (b - 16) % 8;
    return int64_t(8 + m) << (o - 3);
}

// Row stride (floats) of the hub partial-sum scratch for width F: whole 32-byte groups, so that
// vector stores of a last, partial strip stay inside the row.
static inline int64_t gnn_partial_ld(int64_t F) { return (F + 7) / 8 * 8; }

// Share of all gathers that goes to the K most-gathered vertices (from the bucket histogram;
// the boundary bucket is taken pro rata).
double gnn_plan_top_share(const gnn_plan *plan, int64_t K);

// Layout decisions shared by the hot calls and gnn_plan_prepare (which must reserve exactly what
// a later call will use).
struct gnn_layout {
    bool slices_wanted;   // spread column slices over the XCDs
    bool padded_copy;     // gather from a plan-owned copy with rows of an odd number of lines
    int64_t ld_pad;       // row stride of that copy in elements
    // Dense tail: when the last line of a row would hold at most 64 bytes, those columns go into a
    // table of their own with rows of 16-byte groups, packed back to back, so that an L2 line holds
    // the tail of several rows (F = 100 fp32: 3 whole lines per row + a 16-byte tail, 8 rows per
    // line) and the copy's rows are whole lines with nothing wasted.
    int64_t tail_elems;   // columns of the tail table (0: none); the main part has F - tail_elems
    int64_t tail_ld;      // its row stride in elements
    // Slice-major: the main part is stored as one table per 128-byte column slice (line k of every
    // row, rows back to back), because a launch's slice k is only ever read by the XCDs that serve
    // it: their page and DRAM-row footprint shrinks to that table, and no row padding is needed to
    // spread the L2 channels.
    bool slice_major;
    int64_t table_stride; // elements between two slice tables (N * elements per line)
    int64_t main_lines;   // number of slice tables
    int64_t bytes;        // size of the whole copy for N rows
};

// Will calls with this plan serve their long rows as source-blocked pieces (gnn_plan_blocked)?  Known
// once the layout is built; before that, the gate of the automatic choice evaluated on the plan's host
// figures (an explicit gnn_plan_set_blocking counts as yes).
static inline bool gnn_plan_blocks_expected(const gnn_plan *plan, int esz) {
    if (!plan || plan->n_edges <= 0 || plan->n_edges >= int64_t(INT32_MAX)) return false;
    const bool automatic = plan->blocking.min_degree == 0;
    if (esz == 2 && automatic && plan->n_rows < 8 * int64_t(32768)) return false;
    if (plan->blk_decided) return plan->blk_n_pieces > 0;
    if (plan->blocking.min_degree < 0) return false;
    const int64_t min_degree = automatic ? 256 : plan->blocking.min_degree;
    int first_bin = -1;
    for (int i = 0; i < plan->params.n_thresholds; ++i)
        if (plan->params.thresholds[i] == min_degree) first_bin = i + 1;
    if (first_bin < 0 || plan->n_rows - plan->bin_offsets[first_bin] <= 0) return false;
    int64_t long_edges = 0;
    for (int b = first_bin; b < plan->n_bins; ++b) long_edges += plan->bin_edges[b];
    if (long_edges <= 0) return false;
    return !automatic || (plan->n_rows >= 4 * int64_t(32768) && long_edges * 4 >= plan->n_edges);
}

static inline gnn_layout gnn_choose_layout(const gnn_plan *plan, int64_t N, int64_t F, int esz, int64_t ldx,
                                           bool base_line_aligned, int flags, int max_slices, bool allow_tail = false,
                                           bool scaled_source = false, bool blocks_expected = false) {
    gnn_layout L{};
    const int64_t line_elems = 128 / esz;
    const int64_t lines = (F + line_elems - 1) / line_elems;
    const int64_t row_bytes = F * esz;
    // Do column slices pay?  Unsliced, an XCD's 4 MB L2 holds whole rows (32768 / lines of them);
    // sliced, one line each of 32768 rows.  Slicing is used when that wins at least 8 points of
    // the gathers (a power-law graph of a few million vertices: +20..30 points; a 111 M-vertex
    // graph with 2-line rows: ~+2 points, where the extra index reads and the loss of burst
    // locality cost more than the hits bring: 76.2 ms sliced, 74.1 ms without slices).
    L.slices_wanted = !(flags & GNN_FLAG_NO_COLUMN_SLICES);
    if (L.slices_wanted && plan && plan->n_edges > 0 && max_slices == 0) {
        const double gain = gnn_plan_top_share(plan, 32768) - gnn_plan_top_share(plan, 32768 / (lines > 0 ? lines : 1));
        L.slices_wanted = gain >= 0.08;
    }
    // Column slices make XCD k read the same lines (k, k+S, ...) of every row.  With a row stride
    // of an even number of lines those addresses share their low line-index bits and crowd a few
    // of the XCD's 16 L2 channels (measured at F=256, 8 slices: 15.4 ms with 8-line rows, 12.5 ms
    // with 9-line rows).  An odd stride spreads them over all channels, so the padded copy always
    // has one; rows that are not whole lines, and line-aligned rows with an even stride when the
    // gather (E rows) dwarfs the copy (N rows: >= 16 edges per vertex for rows of >= 512 bytes,
    // >= 128 for shorter ones), are copied when slices are wanted.  So are fp32 rows that carry a
    // factor as gathered rows (scaled_source: MEAN / SAGE_GCN backward, weight-less GCN): the copy
    // multiplies it in, which saves the per-edge factor stream and multiply (2.45 M vertices, 50
    // edges each, backward MEAN: F=96 4.98 -> 4.53 ms, F=224 11.6 -> 10.6; 233 K vertices, 490 edges
    // each: F=96 3.00 -> 2.48, F=224 6.85 -> 5.60).
    const bool lines_ok = (ldx % line_elems == 0) && base_line_aligned;
    const bool even_stride = lines_ok && (ldx / line_elems) % 2 == 0;
    const bool big = N * row_bytes >= (int64_t(32) << 20);  // well beyond the L2s: the layout decides the hit rate
    const bool dense_enough = plan && plan->n_edges >= 16 * N;  // the copy (N rows) is small next to the gather (E rows)
    const bool pays_at_any_size = dense_enough && N * row_bytes >= (int64_t(1) << 20);
    const bool folds_factor = scaled_source && esz == 4;
    // More than one line.  Rows that are not whole lines are copied whatever the size of the matrix
    // (in place they are gathered with narrow loads and straddle lines: 233 K vertices, 490 edges
    // each, F=33 fp32 3.16 -> 1.53 ms, F=65 bf16 8.16 -> 1.65), and so are rows that carry a factor;
    // line-aligned rows with an even stride only when the matrix is large and slices are wanted.
    bool worth_it = row_bytes > 128 &&
                    ((!lines_ok && pays_at_any_size) || (folds_factor && pays_at_any_size) ||
                     (big && L.slices_wanted && even_stride && plan && plan->n_edges >= (row_bytes >= 512 ? 16 : 128) * N) ||
                     // the long rows as source-blocked pieces need the slice tables: whatever the stride, the copy
                     // (N rows) buys the pieces (2.45 M vertices, 50 edges each, forward MEAN: F=96 4.42 in place,
                     // 3.53 ms copied; F=64 3.09 / 2.45; F=160 7.48 / 5.81)
                     (blocks_expected && big && L.slices_wanted && allow_tail && lines <= 256));
    // Rows of at most one line are copied into rows of the next power of two bytes (16 ... 128), in
    // rank order: no row straddles two lines, the most-gathered rows share lines (up to 8 per
    // line), and 16-byte loads apply.  Worth it when rows would straddle in place (F = 24: 96-byte
    // rows) or carry a factor that the copy folds in, and for large matrices when they are at most
    // 64 bytes (rank order packs the hot rows).
    int64_t narrow_bytes = 16;
    while (narrow_bytes < row_bytes) narrow_bytes *= 2;
    if (lines == 1) {
        const int64_t stride_bytes = ldx * esz;
        const bool in_place_ok = base_line_aligned && stride_bytes <= 128 && (stride_bytes & (stride_bytes - 1)) == 0;
        worth_it = (!in_place_ok && pays_at_any_size) || (folds_factor && pays_at_any_size) ||
                   (row_bytes <= 64 && big && dense_enough);
    }
    L.padded_copy = plan && !(flags & GNN_FLAG_NO_PADDED_COPY) && (worth_it || (flags & GNN_FLAG_FORCE_PADDED_COPY));
    L.ld_pad = lines == 1 ? narrow_bytes / esz : (lines | 1) * line_elems;
    L.tail_elems = 0;
    L.tail_ld = 0;
    const int64_t rest = F % line_elems;
    // A dense table for a short last line saves its padding and packs eight rows' tails into a line, but it
    // is a launch of its own over all rows; where the long rows are source-blocked pieces the last line
    // does better as one more slice of whole lines, which the pieces serve like the others (2.45 M
    // vertices: F=100 4.84 -> 4.74 ms, F=112 5.08 -> 4.55; 233 K vertices F=100 2.63 -> 2.44).  Packed
    // copies kept by a caller never have the tail table (GNN_FLAG_NO_DENSE_TAIL): their size must not depend
    // on the plan.
    const bool dense_tail = allow_tail && !blocks_expected && !(flags & GNN_FLAG_NO_DENSE_TAIL);
    if (dense_tail && L.padded_copy && L.slices_wanted && lines >= 2 && lines <= 256 && rest > 0 && rest * esz <= 64) {
        const int64_t group = 16 / esz;
        L.tail_elems = rest;
        L.tail_ld = (rest + group - 1) / group * group;
        L.ld_pad = ((lines - 1) | 1) * line_elems;
    }
    L.main_lines = L.tail_elems > 0 ? lines - 1 : lines;
    L.slice_major = allow_tail && L.padded_copy && L.slices_wanted && lines >= 2 && lines <= 256 &&
                    !(flags & GNN_FLAG_NO_SLICE_TABLES);
    L.table_stride = 0;
    if (L.slice_major) {
        L.ld_pad = line_elems;
        L.table_stride = N * line_elems;
        L.bytes = N * (L.main_lines * line_elems + L.tail_ld) * esz;
    } else {
        L.bytes = N * (L.ld_pad + L.tail_ld) * esz;
    }
    return L;
}

// Makes plan->padded at least `bytes` large (allocation on growth).
int gnn_plan_padded(gnn_plan *plan, int64_t bytes);

// The plan's index copy with cold sources flagged in bit 31, or nullptr when cold hints do not pay
// for this graph (see plan.hip).  force: build it whatever the graph (tests).  Builds on first use
// (allocation).
int gnn_plan_cold_indices(gnn_plan *plan, const int32_t *indices, bool force, hipStream_t stream, const int32_t **out);

// Rank layout (see gnn_plan): the vertex ranks and the rank-mapped, cold-flagged index copy.
// force_cold: flag the sources outside the warmest quarter whatever the graph (tests).
struct gnn_rank_layout {
    const int32_t *rank;       // [N]
    const int32_t *indices;    // [E] rank-mapped, cold-flagged, in plan order
    const int64_t *p_indptr;   // [N+1]
    const int64_t *p_chunks;   // [n_chunks * 4]
    bool cold_pays;            // the graph is in the regime where non-temporal loads of cold rows pay
};
int gnn_plan_rank_indices(gnn_plan *plan, const void *indptr, const int32_t *indices, bool force_cold, hipStream_t stream,
                          gnn_rank_layout *out);

// rank[v] = position of vertex v by descending count, ties by ascending id (graph.hip).
int gnn_rank_by_count(const int32_t *counts, int64_t N, int32_t *rank, hipStream_t stream);

// mode: 1 = reciprocal, 2 = reciprocal square root, 3 = reciprocal of (count + 1).
// Builds the array on first use (allocation).
// out[e] = fE[(edge_ids ? edge_ids[e] : e) * lde] for the plan's n_edges edges, into a plan-owned
// array (allocated on first use, refilled by every call).
int gnn_plan_edge_operand(gnn_plan *plan, const float *fE, int64_t lde, const int64_t *edge_ids, hipStream_t stream,
                          const float **out);
int gnn_plan_edge_scale(gnn_plan *plan, const int32_t *indices, int mode, hipStream_t stream, const float **out);

// ---- producer-side layout ----
// Where a kernel that PRODUCES a matrix (the dense product of a layer, the masked output gradient)
// writes it when the next step is an aggregation that would otherwise copy it into the plan's layout
// first: directly into that layout -- one table per 128-byte column slice, rows by descending gather
// count, a dense table for a short last line, the factor the rows carry as gathered rows multiplied
// in.  fp32 only.  Element (v, j) of the matrix goes to
//     j <  main_cols:  base[(j / 32) * table_stride + rank[v] * 32 + j % 32]
//     j >= main_cols:  tail[rank[v] * tail_ld + (j - main_cols)]
// times gnn_row_factor(scale_mode, counts[v]).
struct gnn_packed_target {
    bool active;            // false: the aggregation of this plan / width gathers rows where they lie (write them plainly)
    float *base;
    int64_t table_stride;
    int32_t main_cols;
    float *tail;
    int64_t tail_ld;
    const int32_t *rank;
    const int32_t *counts;
    int32_t scale_mode;     // 0 none, 1 reciprocal, 2 reciprocal square root, 3 reciprocal of (count + 1)
};
__host__ __device__ static inline float gnn_row_factor(int mode, int64_t count) {
    if (mode == 3) return 1.0f / static_cast<float>(count + 1);
    const float d = static_cast<float>(count > 1 ? count : 1);
    if (mode == 1) return 1.0f / d;
    if (mode == 2) return 1.0f / sqrtf(d);
    return 1.0f;
}
// The target for the matrix that gnn_aggregate_fwd / _bwd (`backward`) with this plan, op and width F would
// gather next (a dense fp32 [N, F] matrix).  Grows the plan's buffers on first use (allocation).
// force: take the layout whatever the size of the graph (tests).
int gnn_packed_target_for(gnn_plan *plan, const void *indptr, const int32_t *indices, int64_t N, int64_t F, int op, bool backward,
                          bool force, hipStream_t stream, gnn_packed_target *out);
// The aggregation over a matrix that a producer has written into that target (no copy; `force` as above).
int gnn_aggregate_prepacked(const void *indptr, const int32_t *indices, void *out, int64_t N, int64_t F, int op,
                            const gnn_opts *opts, bool backward, bool force, const float *bias, int relu);

// gnn_aggregate_fwd with a fused epilogue: Y = act(aggregate(X) + bias), act = rectifier if relu.
int gnn_aggregate_fwd_epilogue(const void *indptr, const int32_t *indices, const void *X, void *Y, int64_t N, int64_t F,
                               int op, const gnn_opts *opts, const float *bias, int relu);

// ---- work distribution shared by the aggregation kernels (aggregate.hip, ap.hip) ----
// A launch serves all degree bins of a plan at once: the workgroup index is looked up in a small
// table of bins (heaviest work first).  A bin holds rows (64 >> log2_g rows per wavefront, each row
// group being 2^(log2_g - log2_sr) column lanes x 2^log2_sr edge slots) or hub pieces (one per
// wavefront).
enum gnn_bin_kind : int32_t { GNN_BIN_ROWS = 0, GNN_BIN_HUB_PIECES = 1 };

struct gnn_bin_desc {
    int64_t first_block;  // first workgroup index of this bin (before any slice interleaving)
    int64_t item_begin;   // offset into row_perm (rows) or into the piece list (hub pieces)
    int64_t n_items;      // rows or pieces
    int32_t log2_g;       // lanes per row group
    int32_t log2_sr;      // edge slots per group
    int32_t kind;
    int32_t pad;
};

constexpr int GNN_WAVES_PER_BLOCK = 4;  // 256-thread workgroups

// Fills `bins` for a launch whose row groups have 2^log2_c column lanes; returns the number of
// workgroups.  plan == nullptr: all N rows in one bin, whole wavefronts per row.
// first_excluded_bin: rows of bins >= it (and the hub pieces) are left out (they are served as source-blocked pieces).
static inline int64_t gnn_fill_bins(gnn_bin_desc *bins, int32_t *n_bins, const gnn_plan *plan, int64_t N, int log2_c,
                                    int first_excluded_bin = INT32_MAX) {
    const int max_log2_sr = 6 - log2_c;
    int64_t next_block = 0;
    int nb = 0;
    auto add_bin = [&](int kind, int64_t begin, int64_t n_items, int log2_sr) {
        if (n_items <= 0) return;
        gnn_bin_desc &d = bins[nb++];
        d.first_block = next_block;
        d.item_begin = begin;
        d.n_items = n_items;
        d.kind = kind;
        d.log2_sr = log2_sr;
        d.log2_g = kind == GNN_BIN_HUB_PIECES ? 6 : log2_c + log2_sr;
        d.pad = 0;
        const int64_t items_per_block = int64_t(GNN_WAVES_PER_BLOCK) * (64 >> d.log2_g);
        next_block += (n_items + items_per_block - 1) / items_per_block;
    };
    if (plan) {
        const int last = plan->n_bins - 1;
        const bool has_hub = plan->n_chunks > 0;
        // heaviest work first: hub pieces, then bins from long rows to short rows
        if (has_hub && first_excluded_bin > last) add_bin(GNN_BIN_HUB_PIECES, 0, plan->n_chunks, max_log2_sr);
        for (int bi = last; bi >= 0; --bi) {
            if (bi >= first_excluded_bin) continue;
            if (bi == last && has_hub) continue;  // handled as pieces (+ finalize)
            const int64_t lo = bi == 0 ? 0 : plan->params.thresholds[bi - 1];
            // Edge slots per row: enough that the shortest row of the bin still takes ~16 steps
            // (several batches of loads per group), so short rows share a wavefront (64/G rows
            // each) and only long rows get a whole wavefront.
            int lsr = 0;
            while (lo > 1 && (int64_t(2) << lsr) <= lo) ++lsr;  // floor(log2(lo))
            lsr -= 4;
            if (lsr < 0) lsr = 0;
            if (lsr > max_log2_sr) lsr = max_log2_sr;
            add_bin(GNN_BIN_ROWS, plan->bin_offsets[bi], plan->bin_offsets[bi + 1] - plan->bin_offsets[bi], lsr);
        }
    } else {
        add_bin(GNN_BIN_ROWS, 0, N, max_log2_sr);
    }
    *n_bins = nb;
    return next_block;
}

// Copies an fp32 [N, F] matrix with row stride ld_src into rows of stride ld_dst (elements).
int gnn_pad_rows_f32(const float *src, int64_t ld_src, float *dst, int64_t ld_dst, int64_t N, int64_t F, hipStream_t stream);

// gnn_matmul on a typed stream (shared by the C entry point and the layer calls).
// packed: write the result into a producer-side layout instead of C (C may then be nullptr; M = the plan's rows).
// Rectifier gate of a layer's backward pass folded into the product's operand loads: an element of the
// operand counts as 0 where the gate matrix (same shape and strides) is not positive.  a_gate needs
// trans_a == 0 (dZ = G W^T, with W^T given either way), b_gate and colsum need trans_a != 0 and trans_b == 0
// (dW = Z^T G).  colsum: room for colsum_planes planes of N floats; the call writes n_planes of them
// (the column sums of the gated B over each part of the split reduction, to be added in plane order).
struct gnn_gemm_fold {
    const float *a_gate;
    const float *b_gate;
    float *colsum;
    int64_t colsum_planes;
    int64_t n_planes;  // out
};

int gnn_matmul_impl(const float *A, int64_t lda, int trans_a, const float *B, int64_t ldb, int trans_b, float *C, int64_t ldc,
                    int64_t M, int64_t N, int64_t K, const float *bias, int relu, void *workspace, int64_t workspace_bytes,
                    hipStream_t stream, const gnn_packed_target *packed = nullptr, gnn_gemm_fold *fold = nullptr);

static inline int gnn_ilog2_ceil(int64_t x) {
    int l = 0;
    while ((int64_t(1) << l) < x) ++l;
    return l;
}
