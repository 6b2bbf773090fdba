/*
 * gnnagg -- neighbour aggregation for full-batch GNN training on one MI355X.
 *
 * C ABI of libgnnagg.so.  Plain pointers and sizes only; every array argument
 * is a DEVICE pointer unless a comment says "host".  The library never frees
 * or keeps a caller's buffer beyond the stream work of the call it was passed
 * to.  No exception or abort crosses this boundary: every call returns a
 * gnn_status; gnn_status_string() names it.
 *
 * Graph convention (Section 4.1 of the DistGNN paper): the adjacency matrix is
 * stored in CSR by DESTINATION.  Row v of (indptr, indices) lists the sources
 * u of the edges u->v; features are pulled from the sources and reduced into
 * the destination, one owner per output row.
 *
 * Preconditions that the hot calls do NOT check (gnn_validate_csr does):
 * indptr[0] == 0, indptr non-decreasing, 0 <= indices[e] < N.
 */
#ifndef GNNAGG_H
#define GNNAGG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GNN_API __attribute__((visibility("default")))

typedef enum gnn_status {
    GNN_OK = 0,
    GNN_ERR_INVALID_ARG = 1, /* null required pointer, negative size, unknown enum, ld < F, misaligned base */
    GNN_ERR_UNSUPPORTED = 2, /* valid request this build cannot serve (e.g. an op that needs a plan, without one) */
    GNN_ERR_ALLOC = 3,       /* device or host allocation failed (plan creation / workspace growth only) */
    GNN_ERR_LAUNCH = 4,      /* the HIP runtime reported an error at launch or copy */
    GNN_ERR_INVALID_GRAPH = 5, /* gnn_validate_csr found a violated precondition */
    GNN_ERR_SCRATCH_CAPACITY = 6 /* gnn_aggregate_fwd_noalloc: the hub partial sums of this plan and width
                                    do not fit the library's fixed scratch array */
} gnn_status;

/* Reduce variants.  All are sum-reductions over the in-neighbours (Table 1:
 * reducer "sum", message "copylhs", or "mul" by a scalar edge feature when
 * edge_w is given); they differ in the scaling:
 *   SUM      Y[v] = sum_e c_e X[u_e]                c_e = edge_w[e] or 1
 *   MEAN     SUM divided by the row length din[v] (stored edges; empty row -> 0)
 *   GCN_SYM  c_e = 1/sqrt(max(dout[u],1) * max(din[v],1)) when edge_w == NULL;
 *            with edge_w the weights are taken as given (same as SUM).
 *   SAGE_GCN the aggregator of the paper's own runs (Section 6.1): the sum, plus the
 *            vertex's own vector, divided by din[v] + 1:
 *            Y[v] = (sum_e c_e X[u_e] + X[v]) / (din[v] + 1); the backward call computes the
 *            adjoint dX[u] = sum_{e'} c_e' dY[v_e'] / (din[v_e'] + 1) + dY[u] / (din[u] + 1)
 *            and needs a plan (for din). */
typedef enum gnn_op { GNN_SUM = 0, GNN_MEAN = 1, GNN_GCN_SYM = 2, GNN_SAGE_GCN = 3 } gnn_op;

typedef enum gnn_dtype { GNN_F32 = 0, GNN_BF16 = 1 } gnn_dtype;

typedef struct gnn_plan gnn_plan; /* opaque; owns its device buffers */

/* Options of the hot calls.  Zero-initialise, then set what differs. */
typedef struct gnn_opts {
    int32_t dtype;         /* gnn_dtype of X and Y (same for both).  Accumulation is always fp32;
                              BF16 output is rounded to nearest-even once, at the store. */
    int32_t indptr_is_64;  /* 0: indptr is int32_t[N+1];  1: int64_t[N+1] */
    int64_t ldx;           /* row stride of the gathered matrix in elements; 0 means F.  Fastest: a
                              128-byte-aligned base and a stride that is an ODD multiple of 128 bytes
                              (e.g. 288 floats for F = 256): rows are then gathered in place, slice by
                              slice, with all L2 channels in use; other layouts of large matrices are
                              first copied into such rows (plan-owned buffer) when a plan is given */
    int64_t ldy;           /* row stride of the output matrix in elements; 0 means F */
    void *stream;          /* hipStream_t to enqueue on; NULL = the null stream */
    gnn_plan *plan;        /* degree-binning plan OF THE GRAPH PASSED IN THE SAME CALL (forward plan
                              for _fwd, plan of the transposed graph for _bwd); NULL = un-binned
                              wavefront-per-row kernel, no hub splitting.  A hot call may grow
                              plan-owned buffers on first use (see gnn_plan_prepare); two calls
                              sharing one plan must not overlap in time. */
    void *workspace;       /* optional device scratch for hub-row partial sums; NULL = plan-owned
                              scratch, grown (allocation!) on the first call that needs more */
    int64_t workspace_bytes;
    int32_t flags;         /* bit set of GNN_FLAG_*; 0 = defaults */
    int32_t max_slices;    /* upper bound on the number of XCD column slices (1, 2, 4 or 8); 0 = automatic */
} gnn_opts;

/* Do not spread column slices of line-aligned rows over the XCDs (for A/B measurements). */
#define GNN_FLAG_NO_COLUMN_SLICES 1
/* Gather from the caller's matrix even when its rows are not whole 128-byte lines (default: a
 * call with a plan copies such a matrix into plan-owned padded rows first, when it is large). */
#define GNN_FLAG_NO_PADDED_COPY 2
/* Take the padded-copy route whenever a plan is given, whatever the size and alignment (tests). */
#define GNN_FLAG_FORCE_PADDED_COPY 4

/* The caller guarantees that elements F .. ldx-1 of every gathered row are readable (their values
 * are ignored): wide loads may then be used for widths that are not a multiple of 4 (2 for bf16:
 * 8) when ldx is. */
#define GNN_FLAG_PADDED_ROWS 8

/* Cold hints: sliced launches on a large power-law graph fetch the rows of rarely gathered sources
 * with non-temporal loads (the plan keeps a copy of the index array with those sources flagged,
 * 4 bytes per edge, built on first use or by gnn_plan_prepare).  NO: never; FORCE: whatever the
 * graph and layout (tests).  Results do not depend on it. */
#define GNN_FLAG_NO_COLD_HINTS 16
#define GNN_FLAG_FORCE_COLD_HINTS 32
/* Keep the plan-owned padded copy in vertex order (default: rows stored by descending gather
 * count, gathered through a rank-mapped copy of the index array; 4 bytes per edge and per vertex
 * of plan memory).  For A/B measurements; results do not depend on it. */
#define GNN_FLAG_NO_RANK_ORDER 64
/* Keep the plan-owned padded copy row-major (default for sliced launches: one table per 128-byte
 * column slice).  For A/B measurements; results do not depend on it. */
#define GNN_FLAG_NO_SLICE_TABLES 128

/* Do not process the long rows as source-blocked pieces (see gnn_blocking_params).  For A/B
 * measurements; results agree within rounding (the order of the additions differs). */
#define GNN_FLAG_NO_SOURCE_BLOCKS 256
/* Where the long rows are processed as source-blocked pieces, the launches over the short rows run
 * beside them on a second, library-owned stream (default priority; joined before the call's last
 * kernels, so the caller sees one stream; under stream capture that stream joins the capture for the
 * length of the call).  The library has one such stream per device: calls of different host threads
 * queue up on it, and two threads that capture graphs at the same time must set NO.  NO: everything
 * on the caller's stream, one launch after the other (also for A/B measurements).  Results do not
 * depend on it. */
#define GNN_FLAG_NO_SHORT_ROW_OVERLAP 512
/* A plan-owned copy in slice tables normally keeps a last line of at most 64 bytes in a dense table
 * of its own (16-byte groups back to back, eight rows to a line, gathered by a launch of its own),
 * except where the long rows are source-blocked pieces: there that line is one more table of whole
 * lines, which the pieces serve like the others.  NO: always the table of whole lines. */
#define GNN_FLAG_NO_DENSE_TAIL 1024

/* Degree-binning parameters.  thresholds t[0] < ... < t[k-1], all > 0, cut the
 * row-length axis into k+1 bins, bin(v) = #{i : t[i] <= deg(v)}.  If
 * hub_chunk > 0 the rows of the LAST bin are "hub" rows: each is cut into
 * pieces of hub_chunk consecutive edges that different wavefronts reduce, and a
 * second kernel adds the pieces in a fixed order (deterministic, no float
 * atomics).  NULL params = defaults (gnn_plan_default_params). */
#define GNN_MAX_THRESHOLDS 15
typedef struct gnn_plan_params {
    int32_t n_thresholds;
    int64_t thresholds[GNN_MAX_THRESHOLDS];
    int64_t hub_chunk;
} gnn_plan_params;

/* Source blocking of the long rows (Section 4.2 blocks the SOURCE vertices so that a block of f_V
 * stays in cache while all destination rows sweep over it; here only the rows of at least
 * `min_degree` edges take part, cut into pieces along blocks of source vertices ordered by
 * descending gather count, and the pieces of one block run side by side).  All zero = automatic. */
typedef struct gnn_blocking_params {
    int64_t min_degree;      /* rows this long are cut into pieces; must be one of the plan's thresholds.  < 0: never block */
    int64_t hot_lines;       /* sources in block 0 (the most-gathered ones) */
    int64_t block_lines;     /* sources per further block */
    int64_t max_piece;       /* edges per piece at most */
    int64_t rest_min_count;  /* sources gathered fewer times than this share one last block; 0 .. 16 or a boundary of
                                the plan's count histogram above that: 18, 20, .. 32, 36, 40, .. 64, 72, .. (8 per octave) */
} gnn_blocking_params;

/* ---------------------------------------------------------------- hot path */

/* Forward aggregation (Section 4.1, Algorithm 1; equals the sparse-times-dense
 * product of Section 2.1):
 *     Y[v, 0:F] = scale_v * sum_{e in row v} c_e * X[indices[e], 0:F]
 * indptr   [N+1] int32 or int64 (opts->indptr_is_64), CSR by destination
 * indices  [E] int32 source ids, E = indptr[N]
 * edge_w   [E] fp32 in CSR edge order, or NULL
 * X        [N, ldx] gathered matrix, Y [N, ldy] output; fp32 or bf16 per opts->dtype
 * Y is OVERWRITTEN (rows without edges become +0); X and Y must not overlap.
 * Base pointers must be aligned to 16 bytes when the row stride in bytes is a
 * multiple of 16 (8 / 4 / 2 likewise); otherwise narrower loads are used.
 * Asynchronous: returns after enqueueing on opts->stream.  N == 0 or F == 0 is
 * GNN_OK and does nothing.  opts == NULL means all defaults.
 * MEAN needs no plan; GCN_SYM without edge_w needs a plan (it holds dout). */
GNN_API int gnn_aggregate_fwd(const void *indptr, const int32_t *indices, const float *edge_w,
                      const void *X, void *Y, int64_t N, int64_t F, int op, const gnn_opts *opts);

/* gnn_aggregate_fwd for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same result as
 * gnn_aggregate_fwd called with GNN_FLAG_NO_PADDED_COPY | GNN_FLAG_NO_COLD_HINTS, but the call
 * never allocates, frees or grows anything, on the device or in a plan:
 *   - the partial sums of the hub rows go into a fixed array of GNN_NOALLOC_SCRATCH_BYTES that is
 *     part of the library's device code (every GPU the library runs on holds one until the process
 *     ends); a plan and width that need more (gnn_plan_workspace_bytes(plan, F)) are rejected with
 *     GNN_ERR_SCRATCH_CAPACITY before anything is enqueued; opts->workspace is ignored;
 *   - rows are gathered from X where they lie (no plan-owned copy of X or of the index array);
 *   - GNN_GCN_SYM without edge_w reads the plan's per-edge factor stream, which must exist already
 *     (gnn_plan_prepare with GNN_GCN_SYM), else GNN_ERR_UNSUPPORTED.
 * All calls on one GPU share that GPU's array, whatever their stream or plan: calls that overlap
 * in time on one GPU race on it and must be ordered by the caller.  The array keeps the last
 * call's contents; every element that is read has been written by the same call first. */
#define GNN_NOALLOC_SCRATCH_BYTES (32 << 20)
GNN_API int gnn_aggregate_fwd_noalloc(const void *indptr, const int32_t *indices, const float *edge_w,
                      const void *X, void *Y, int64_t N, int64_t F, int op, const gnn_opts *opts);

/* Backward aggregation: the adjoint of the forward map over the transposed
 * graph (the paper only implies it, Section 6.3 "Memory"):
 *     dX[u, 0:F] = sum_{e' in transposed row u} c_e' * dY[indices_t[e'], 0:F]
 * indptr_t / indices_t / edge_w_t describe the TRANSPOSED graph (CSR by
 * source; gnn_transpose_csr builds them).  c_e' carries the same factors as in
 * the forward pass: for MEAN 1/din[v] of the GATHERED vertex v, for GCN_SYM
 * without weights 1/sqrt(max(dout[u],1)*max(din[v],1)).  MEAN and weight-less
 * GCN_SYM therefore need opts->plan (a plan of the transposed graph, which
 * holds din as its column counts); without one they return
 * GNN_ERR_UNSUPPORTED.  No gradient with respect to edge weights is produced.
 * Everything else as for gnn_aggregate_fwd. */
GNN_API int gnn_aggregate_bwd(const void *indptr_t, const int32_t *indices_t, const float *edge_w_t,
                      const void *dY, void *dX, int64_t N, int64_t F, int op, const gnn_opts *opts);

/* Packed copies that the caller keeps (Section 3: full-batch training aggregates the SAME input
 * features in every epoch).  A call on a large graph first copies the gathered matrix into the
 * plan's layout: one table per 128-byte column slice (the last one padded to whole lines), rows
 * ordered by descending gather count.  A caller whose matrix does not change between calls makes
 * that copy once, into a buffer of its own, and gathers from it.
 *
 * gnn_packed_bytes: size of the copy of an [N, F] matrix; 0 when F is at most one line of 128
 *   bytes or more than 256 lines (such rows are not laid out as tables) or an argument is invalid.
 * gnn_pack_rows: writes the copy of X (row stride opts->ldx, 0 = F) into `packed` (device memory,
 *   aligned to 128 bytes, packed_bytes >= gnn_packed_bytes, else GNN_ERR_INVALID_ARG).  `op` and
 *   `backward` must be those of the calls that will gather from it: where the gathered rows carry
 *   a factor (backward GNN_MEAN and GNN_SAGE_GCN, weight-less GNN_GCN_SYM) an fp32 copy holds the
 *   rows already multiplied by it.  Needs opts->plan of the graph the calls run on (the row order
 *   is that plan's), else GNN_ERR_UNSUPPORTED; a graph without edges is GNN_ERR_UNSUPPORTED too.
 * gnn_aggregate_packed: gnn_aggregate_fwd (backward == 0: the arrays describe the graph) or
 *   gnn_aggregate_bwd (backward != 0: the transposed graph) reading `packed` in place of the
 *   matrix; same result as those calls with GNN_FLAG_FORCE_PADDED_COPY | GNN_FLAG_NO_DENSE_TAIL
 *   and max_slices = 8, bit for bit, without their copy.  opts->ldx is ignored; the layout flags
 *   of opts are overridden.
 * The buffer stays the caller's; the library keeps no reference to it after the call's work has
 * run. */
GNN_API int64_t gnn_packed_bytes(int64_t N, int64_t F, int dtype);
GNN_API int gnn_pack_rows(const void *indptr, const int32_t *indices, const void *X, void *packed,
                      int64_t packed_bytes, int64_t N, int64_t F, int op, int backward, const gnn_opts *opts);
GNN_API int gnn_aggregate_packed(const void *indptr, const int32_t *indices, const float *edge_w,
                      const void *packed, int64_t packed_bytes, void *Y, int64_t N, int64_t F, int op,
                      int backward, const gnn_opts *opts);

/* ------------------------------------- general aggregation primitive (fp32) */

/* The operator table of Section 4.1 (Table 1).  x = f_V[u, j] of the source vertex, y = f_E[e, j]
 * of the edge; copylhs ignores y, copyrhs ignores x. */
typedef enum gnn_binop {
    GNN_BIN_ADD = 0, GNN_BIN_SUB = 1, GNN_BIN_MUL = 2, GNN_BIN_DIV = 3, GNN_BIN_COPY_LHS = 4, GNN_BIN_COPY_RHS = 5
} gnn_binop;
typedef enum gnn_reduce { GNN_RED_SUM = 0, GNN_RED_MAX = 1, GNN_RED_MIN = 2 } gnn_reduce;

/* Options of the gnn_ap_* calls.  Zero-initialise, then set what differs. */
typedef struct gnn_ap_opts {
    int32_t indptr_is_64;     /* as in gnn_opts */
    int32_t edge_width;       /* columns of f_E in use: 0 or d = one per feature column; 1 = one scalar
                                 per edge that serves every column */
    int64_t ldv, lde, ldo;    /* row strides in floats of f_V, f_E and f_O (and of their gradients);
                                 0 = d, edge_width, d */
    const int64_t *edge_ids;  /* [E] device, or NULL: the row of f_E that the edge at CSR position e
                                 uses (NULL: row e).  A transposed graph passes the `perm` of
                                 gnn_transpose_csr here to keep addressing the original edge rows.
                                 Must not name a row twice when an edge gradient is written. */
    void *stream;
    gnn_plan *plan;           /* plan of the graph passed in the same call, or NULL (no binning) */
    int32_t flags;            /* GNN_FLAG_NO_COLUMN_SLICES / NO_PADDED_COPY / FORCE_PADDED_COPY, as in gnn_opts:
                                 gather-bound forward calls (no full-width edge operand, d % 4 == 0, a plan)
                                 use the layout of the sum-only hot path */
    int32_t max_slices;       /* as in gnn_opts; 0 = automatic */
} gnn_ap_opts;

/* Algorithm 1 with any operator pair of Table 1:
 *     f_O[v, j] = reduce over the edges e = (u -> v) of row v of  binop(f_V[u, j], f_E[e, j])
 * f_V [*, ldv] (not read by copyrhs, may be NULL then), f_E [*, lde] (not read by copylhs),
 * f_O [N, ldo] is overwritten.  The reduction starts from the identity of `reduce`; a row without
 * edges yields 0.  sum accumulates in fp32.  max / min: every message is one correctly rounded
 * fp32 operation, so the result is exact; arg_e (optional, int32 [N, d], dense) receives the CSR
 * position of the winning edge of every (v, j) -- the lowest position among equals, -1 for an
 * empty row -- and must be NULL for sum.  NaN inputs give an unspecified winner.  max / min need
 * E <= INT32_MAX.  16-byte loads are used when d, the strides and the base addresses allow,
 * scalar ones otherwise; a gather-bound call on a large graph with a plan is then staged through
 * plan-owned padded rows (1.1-1.2x the time of the next multiple of 4).  Hub rows use plan-owned
 * scratch (grown on first use: allocation).
 * copylhs / sum and mul / sum with a scalar f_E are what gnn_aggregate_fwd computes with GNN_SUM
 * (plain or weighted) and run on that path, with its layouts; a scalar f_E that is strided or
 * addressed through edge_ids is first gathered into a plan-owned array of E floats (allocated on
 * first use) when a plan is given.
 * Asynchronous on opts->stream. */
GNN_API int gnn_ap_fwd(const void *indptr, const int32_t *indices, const float *fV, const float *fE,
                       float *fO, int32_t *arg_e, int64_t N, int64_t d, int binop, int reduce,
                       const gnn_ap_opts *opts);

/* Gradient of sum_{v,j} dO[v,j] f_O[v,j] with respect to f_V for reduce = sum (the paper does not
 * spell out backward passes; this is the derivative of the definition above).  It is the same
 * primitive over the TRANSPOSED graph, gathering dO: copylhs for add / sub / copylhs, mul by f_E
 * for mul, div by f_E for div, zero for copyrhs.  indptr_t / indices_t / opts (plan, edge_ids =
 * perm, or perm composed with the forward edge_ids) describe the transposed graph.  dfV [N, ldv]
 * is overwritten. */
GNN_API int gnn_ap_bwd_vertex(const void *indptr_t, const int32_t *indices_t, const float *dO, const float *fE,
                              float *dfV, int64_t N, int64_t d, int binop, const gnn_ap_opts *opts);

/* The same gradient for reduce = max / min, where only the winning edge of each (v, j) carries
 * gradient: dfV[indices[arg_e[v,j]], j] += dO[v,j] * d(binop)/dx.  Runs over the FORWARD graph's
 * `indices` and the arg_e that gnn_ap_fwd wrote; N*d fp32 atomic adds into dfV [n_vertex_rows, ldv]
 * (zero-filled first), so the summation order, and with it the last bits, vary from run to run. */
GNN_API int gnn_ap_bwd_vertex_arg(const int32_t *indices, const int32_t *arg_e, const float *dO, const float *fE,
                                  float *dfV, int64_t n_vertex_rows, int64_t N, int64_t d, int binop,
                                  const gnn_ap_opts *opts);

/* Gradient with respect to f_E, one output row per edge (the sampled dense-dense product of
 * Section 2.2 when edge_width = 1 and binop = mul: dfE[e] = <dO[v, :], f_V[u, :]>):
 *     dfE[r(e), j] = dO[v, j] * d(binop)/dy          add: 1, sub: -1, mul: x, div: -x / y^2, copyrhs: 1
 * summed over j when edge_width = 1; for max / min (arg_e != NULL) only where arg_e[v, j] == e,
 * zero elsewhere.  Runs over the forward graph; r(e) = edge_ids[e] or e; dfE has f_E's layout
 * (lde) and every row an edge names is overwritten.  copylhs has no edge operand:
 * GNN_ERR_INVALID_ARG. */
GNN_API int gnn_ap_bwd_edge(const void *indptr, const int32_t *indices, const int32_t *arg_e, const float *fV,
                            const float *fE, const float *dO, float *dfE, int64_t N, int64_t d, int binop,
                            const gnn_ap_opts *opts);

/* ------------------------------------------------ dense update of a layer (fp32) */

/* The MLP step that follows the aggregation in every layer (Section 6.3, "Memory": weight
 * matrices f x h1, h1 x h2, h2 x l), on the matrix cores with exact fp32 products:
 *     C[m, n] = act( sum_k opA(A)[m, k] * opB(B)[k, n] + bias[n] ),   act = max(., 0) if relu
 * A is stored [M, K] with row stride lda, or [K, M] when trans_a; B is stored [K, N] with row
 * stride ldb, or [N, K] when trans_b; C [M, ldc] is overwritten; bias [N] or NULL.  All device
 * pointers.  A long reduction with few output tiles (the weight gradient: K = number of vertices)
 * is split into partial products that are added in a fixed order; that needs `workspace` of
 * gnn_matmul_workspace_bytes(M, N, K) bytes (0 for most shapes); without it the call still
 * works, unsplit.  16-byte loads are used when the leading dimensions and bases allow.
 * Asynchronous on `stream`; allocates nothing. */
GNN_API int gnn_matmul(const float *A, int64_t lda, int trans_a, const float *B, int64_t ldb, int trans_b,
                       float *C, int64_t ldc, int64_t M, int64_t N, int64_t K, const float *bias, int relu,
                       void *workspace, int64_t workspace_bytes, void *stream);
GNN_API int64_t gnn_matmul_workspace_bytes(int64_t M, int64_t N, int64_t K);

/* ------------------------------------------- one GraphSAGE layer (fp32) */

/* Options of the layer calls.  Zero-initialise, then set what differs. */
typedef struct gnn_layer_opts {
    int32_t indptr_is_64;
    int32_t relu;        /* 1: rectifier after the bias; 0: identity (a last layer) */
    int32_t order;       /* 0: aggregate first iff F_in <= F_out, else transform first (the two linear
                            steps commute; the narrower rows are gathered); 1 / 2 force either */
    int32_t flags;       /* bit set of GNN_LAYER_*; 0 = defaults */
    void *stream;
    gnn_plan *plan;      /* REQUIRED: plan of the graph passed in the same call (forward plan for _fwd,
                            plan of the transposed graph for _bwd) */
    void *workspace;     /* _bwd only: device scratch of gnn_sage_layer_workspace_bytes(), 16-byte aligned */
    int64_t workspace_bytes;
} gnn_layer_opts;

/* Producer-side layouts: inside a layer the matrix that the aggregation gathers is often produced by the
 * step before it (X W when transforming first; dH masked, or its product with W^T, in the backward
 * pass).  Where the aggregation would first copy that matrix into the plan's layout (large graphs),
 * the producing kernel writes it there directly.  FORCE: whatever the size of the graph (tests);
 * NO: never (A/B measurements).  Results do not depend on it beyond rounding. */
#define GNN_LAYER_FORCE_PRODUCER_LAYOUT 1
#define GNN_LAYER_NO_PRODUCER_LAYOUT 2
/* Backward pass, aggregating first: the masked gradient G = dH where H > 0 is an operand of two
 * products only, so they read dH and H themselves and apply the rectifier while staging the
 * operand, and the weight-gradient product also adds up the bias gradient; G is never written.
 * NO_GATE_FOLD: write G first with a kernel of its own instead (A/B measurements; with a rectifier the
 * workspace must then be N * F_out * 4 + 256 bytes larger than gnn_sage_layer_workspace_bytes says).
 * dW and db are reproducible run to run either way; between the two settings they differ by
 * rounding only. */
#define GNN_LAYER_NO_GATE_FOLD 4

/* One layer of the paper's model: the aggregation (Section 6.1: sum of the in-neighbours' vectors
 * plus the vertex's own, divided by in-degree + 1) followed by the dense update (Section 6.3,
 * "Memory": one weight matrix per layer), with a bias and an optional rectifier (not stated in
 * the paper; the usual GraphSAGE layer):
 *     H[v, :] = act( ((sum_{u->v} X[u, :] + X[v, :]) / (din[v] + 1)) W + b )
 * X [N, F_in], W [F_in, F_out] row-major, bias [F_out] or NULL, H [N, F_out], all dense fp32.
 * `saved` receives what the chosen order materialises, gnn_sage_layer_saved_elems() floats: the
 * aggregated input Z [N, F_in] (aggregate first; the backward call needs it) or the transformed
 * input X W with rows padded to a multiple of 4 floats (transform first; only a temporary).  Asynchronous on opts->stream; the
 * aggregation may grow plan-owned buffers on first use (gnn_plan_prepare with GNN_SAGE_GCN). */
GNN_API int gnn_sage_layer_fwd(const void *indptr, const int32_t *indices, const float *X, const float *W,
                               const float *bias, float *saved, float *H, int64_t N, int64_t F_in, int64_t F_out,
                               const gnn_layer_opts *opts);
/* Gradients of sum_{v,j} dH[v,j] H[v,j]: dW [F_in, F_out], db [F_out] (may be NULL), dX [N, F_in] (may
 * be NULL: a first layer needs none).  The rectifier passes gradient where the stored forward
 * output H is > 0.  indptr_t / indices_t / opts->plan describe the TRANSPOSED graph; `saved` is
 * what the forward call wrote (needed when aggregating first; may be NULL otherwise).  opts->relu
 * and opts->order must be those of the forward call.  Sums over vertices (dW, db) are formed in a
 * fixed order: results are reproducible run to run. */
GNN_API int gnn_sage_layer_bwd(const void *indptr_t, const int32_t *indices_t, const float *X, const float *W,
                               const float *saved, const float *H, const float *dH, float *dX, float *dW,
                               float *db, int64_t N, int64_t F_in, int64_t F_out, const gnn_layer_opts *opts);
GNN_API int64_t gnn_sage_layer_saved_elems(int64_t N, int64_t F_in, int64_t F_out, int order);
GNN_API int64_t gnn_sage_layer_workspace_bytes(int64_t N, int64_t F_in, int64_t F_out, int relu, int order);

/* ------------------------------------------------------- once-per-graph setup */

/* Row pointers of the destination-indexed CSR (Section 4.1 requires the graph
 * in CSR) from a destination array sorted ascending:
 * indptr[v] = #{e : dst_sorted[e] < v}.  indptr_out has N+1 entries of the
 * width indptr_is_64 selects.  E may be 0.  Asynchronous on `stream`. */
GNN_API int gnn_csr_from_sorted_coo(const int32_t *dst_sorted, int64_t E, int64_t N,
                            void *indptr_out, int indptr_is_64, void *stream);

/* Transposed graph (what the backward pass runs over), by a STABLE sort on the
 * source id: inside transposed row u the edges keep their CSR order, so a CSR
 * with ascending neighbours gives ascending destinations.
 * Outputs (caller-allocated): indptr_t [N+1] (same width as indptr),
 * indices_t [E] int32, and optionally perm [E] int64 (perm[e'] = CSR position
 * of transposed edge e'; may be NULL) and edge_w_t [E] = edge_w[perm] (only if
 * edge_w != NULL).  E is read from the device (indptr[N]); the call allocates
 * temporary device memory (about 24 bytes per edge), frees it and is
 * SYNCHRONOUS with respect to `stream`. */
GNN_API int gnn_transpose_csr(const void *indptr, const int32_t *indices, const float *edge_w,
                      int64_t N, int indptr_is_64, void *indptr_t, int32_t *indices_t,
                      int64_t *perm, float *edge_w_t, void *stream);

/* Checks the preconditions of the hot calls on the device (debug aid; reads E
 * back, synchronous).  GNN_OK or GNN_ERR_INVALID_GRAPH. */
GNN_API int gnn_validate_csr(const void *indptr, const int32_t *indices, int64_t N, int64_t E,
                     int indptr_is_64, void *stream);

/* Degree-binning plan of one graph orientation: the GPU replacement for the
 * dynamic scheduling of destination rows in Section 4.2 ("Multithreading").
 * Holds row_perm (rows grouped by bin, ascending row id inside a bin),
 * bin_offsets, the hub-row piece list and the per-vertex column counts
 * (#occurrences of each vertex in `indices`: dout for a forward graph, din for
 * a transposed one).  Synchronous; allocates device memory owned by the plan.
 * params == NULL: defaults.  *out receives the plan. */
GNN_API void gnn_plan_default_params(gnn_plan_params *params /* host, out */);
GNN_API int gnn_plan_create(const void *indptr, const int32_t *indices, int64_t N, int indptr_is_64,
                    const gnn_plan_params *params /* host */, void *stream, gnn_plan **out);
GNN_API void gnn_plan_destroy(gnn_plan *plan);

/* Sizes of what gnn_plan_export would write (host outputs). */
GNN_API int gnn_plan_sizes(const gnn_plan *plan, int64_t *n_rows, int32_t *n_bins, int64_t *n_chunks);
/* Copies the plan to HOST arrays for inspection / bit-exact checks:
 * bin_offsets int64[n_bins+1], row_perm int32[n_rows], chunks int64[n_chunks*3]
 * as (row, e_begin, e_end), col_counts int32[n_rows].  Any may be NULL. */
GNN_API int gnn_plan_export(const gnn_plan *plan, int64_t *bin_offsets, int32_t *row_perm,
                    int64_t *chunks, int32_t *col_counts);
/* Share (0..1) of all gathers that goes to the K most-gathered vertices of the plan's graph
 * (from a 256-bucket histogram of the column counts, so accurate to a few percent).  The hot
 * calls use it to decide whether spreading column slices over the XCDs can keep more useful
 * rows in the 4 MB L2 caches; exported for inspection. */
GNN_API double gnn_plan_gather_share(const gnn_plan *plan, int64_t K);
/* Bytes of scratch a hot call with this plan and width F needs (hub partials). */
GNN_API int64_t gnn_plan_workspace_bytes(const gnn_plan *plan, int64_t F);
/* Grow the plan-owned scratch now, so later hot calls do not allocate. */
GNN_API int gnn_plan_reserve(gnn_plan *plan, int64_t F);
/* Everything a later hot call with (op, direction, F) would otherwise allocate on its first
 * use: the scratch of gnn_plan_reserve; the plan-owned per-edge factor stream (4 bytes per edge:
 * 1/din or 1/sqrt(deg) of the gathered vertex) that MEAN backward and weight-less GCN_SYM read
 * instead of one random count lookup per edge; for large matrices whose rows are not whole
 * 128-byte lines (or have an even line stride) the plan-owned copy of the gathered matrix that
 * the hot call fills and gathers from (about N x F elements of `dtype`, rows stored by descending
 * gather count, a short last line kept in a dense table of its own); and the index copy that goes
 * with it (4 bytes per edge + 12 per vertex: source ids mapped to their rank, edge lists in the
 * plan's row order), or -- where no copy of the matrix is made but column slices are used on a
 * large power-law graph -- the index copy with the cold sources flagged.  `indices` is the index
 * array of the plan's graph, and the row pointers the plan was created from must still be alive.
 * backward: 0 for gnn_aggregate_fwd, 1 for gnn_aggregate_bwd. */
GNN_API int gnn_plan_prepare(gnn_plan *plan, const int32_t *indices, int op, int backward, int64_t F,
                             int dtype, void *stream);

/* Sets the source-blocking parameters of a plan (before its first hot call or gnn_plan_prepare;
 * later calls return GNN_ERR_UNSUPPORTED once the layout is built).  NULL = automatic. */
GNN_API int gnn_plan_set_blocking(gnn_plan *plan, const gnn_blocking_params *params /* host */);
/* Declares an edge-weight array static (Section 3: full-batch training runs every layer and epoch over
 * the same graph, and the edge features f_E of Algorithm 1 that normalise it belong to that graph): the plan
 * keeps a copy of `edge_w` (device, fp32, in the CSR order of the plan's graph, as the hot calls take it)
 * in the order its source-blocked pieces read, and hot calls with this plan that pass THE SAME POINTER
 * serve their long rows as pieces, streaming the copy; other weight arrays keep the path without
 * pieces (a piece would read the caller's array at random, 4 bytes per edge).  The copy is made on `stream`
 * now if the plan's layout exists already, else by the first hot call or gnn_plan_prepare that builds it
 * (one allocation of 4 bytes per edge of the long rows).  Call again whenever the array's contents
 * change -- the short rows read the caller's array, the long rows the copy, so a stale copy gives
 * results that mix the two; later hot calls on other streams must be ordered after `stream` by the
 * caller.  NULL unbinds.  The array stays the caller's and must outlive the binding. */
GNN_API int gnn_plan_bind_edge_weights(gnn_plan *plan, const float *edge_w /* device or NULL */, void *stream);
/* Sizes of the source-blocked layout (all 0 when the plan has none, or has not built it yet):
 * rows served as pieces, their edges, pieces, blocks. */
GNN_API int gnn_plan_blocked_sizes(const gnn_plan *plan, int64_t *n_rows, int64_t *n_edges, int64_t *n_pieces,
                                   int32_t *n_blocks);
/* Host copies for bit-exact checks: indices int32[n_edges] (source ranks in block-major piece
 * order), epos uint32[n_edges] (CSR position of each), pieces int32[n_pieces*4] as (begin, length,
 * partial slot, row index within the blocked rows), rowbase uint32[n_rows+1], rank int32[N] (rank of
 * every vertex by descending gather count, ties by ascending id).  Any may be NULL. */
GNN_API int gnn_plan_export_blocked(const gnn_plan *plan, int32_t *indices, uint32_t *epos, int32_t *pieces,
                                    uint32_t *rowbase, int32_t *rank);

/* ---------------------------------------------------------------- utilities */
GNN_API const char *gnn_status_string(int status);

/* Streaming copy of n_bytes (multiple of 16; both pointers 16-byte aligned): the kernel of
 * known traffic that the bench prints as a measured ceiling and that the profiler runs use to
 * calibrate the FETCH_SIZE / WRITE_SIZE counters. */
GNN_API int gnn_calib_copy(const void *src, void *dst, int64_t n_bytes, void *stream);

/* Bare gather of 128-byte lines, a second measured ceiling: `table` holds n_lines lines (128-byte
 * aligned), line_ids [n_ids] uint32 names the lines to fetch (ids beyond the table are clamped to its
 * last line), 8 lanes fetch a line, 16 lines are in flight per lane group; 8,388,608 threads each write
 * one float of `out` (out_elems >= 8,388,608, else GNN_ERR_INVALID_ARG).  Gathers
 * floor(n_ids / 1,048,576 / 16) * 16 lines per lane group (at least 16, else GNN_ERR_INVALID_ARG). */
GNN_API int gnn_calib_gather(const void *table, int64_t n_lines, const uint32_t *line_ids, int64_t n_ids, float *out,
                             int64_t out_elems, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* GNNAGG_H */
