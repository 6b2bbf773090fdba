// One GraphSAGE layer: neighbourhood aggregation followed by the dense update (Section 6.3,
// "Memory": every layer is the aggregation step followed by the MLP operation with one weight
// matrix), with the aggregator of the paper's runs (Section 6.1: sum of the in-neighbours plus the
// vertex's own vector, over in-degree + 1):
//
//     H = act( A^ X W + b ),     A^ = D^-1 (A + I),  D = diag(din + 1)
//
// Both steps are linear, so the cheaper order is taken: aggregate first when F_in <= F_out
// (gather rows of width F_in), transform first otherwise (gather rows of width F_out: the class
// scores of a last layer, or 16 hidden units after 602 input features); in the second case bias
// and rectifier are the epilogue of the aggregation kernel, in the first of the matrix product.
// The backward pass mirrors the order taken:
//     G  = dH where H > 0 (rectifier; the stored forward output decides), db = column sums of G
//     aggregate first:  dW = Z^T G,  dZ = G W^T,  dX = A^^T dZ          (Z = A^ X, stored by forward)
//     transform first:  dP = A^^T G, dW = X^T dP, dX = dP W^T
#include "common.h"

#include <mutex>

namespace {

constexpr int kRowsPerBlock = 128;

// A library-owned side stream per device (default priority, created on first use, kept until
// the process ends): the weight-gradient product, which depends only on G, runs there while the
// main stream does the input-gradient product and the gather-bound backward aggregation.
hipStream_t side_stream() {
    static std::mutex mu;
    static hipStream_t streams[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (!streams[dev] && hipStreamCreateWithFlags(&streams[dev], hipStreamNonBlocking) != hipSuccess) streams[dev] = nullptr;
    return streams[dev];
}

// G = dH where H > 0 (else 0; plain copy without a rectifier) for a block of rows, written with row
// stride ldg when G != nullptr, plus the block's column sums.  A thread owns one column and every
// (256 / cols)-th row of the block; the row lanes are added through LDS in a fixed order, so the
// sums are reproducible.  cols = power of two >= F, at most 256 (wider F: several column passes).
// pk.active: G goes into a producer-side layout (the tables the backward aggregation gathers from) instead.
__global__ void __launch_bounds__(256) mask_colsum_kernel(const float *__restrict__ H, const float *__restrict__ dH,
                                                          float *__restrict__ G, int64_t ldg, float *__restrict__ partial,
                                                          int64_t N, int F, int relu, int log2_cols, const gnn_packed_target pk) {
    __shared__ float red[256];
    const int cols = 1 << log2_cols;
    const int row_lanes = 256 >> log2_cols;
    const int jl = threadIdx.x & (cols - 1), rl = threadIdx.x >> log2_cols;
    const int64_t r0 = int64_t(blockIdx.x) * kRowsPerBlock;
    const int64_t r1 = r0 + kRowsPerBlock < N ? r0 + kRowsPerBlock : N;
    for (int j0 = 0; j0 < F; j0 += cols) {
        const int j = j0 + jl;
        float s = 0.0f;
        if (j < F) {
            for (int64_t r = r0 + rl; r < r1; r += row_lanes) {
                float g = dH[r * F + j];
                if (relu) g = H[r * F + j] > 0.0f ? g : 0.0f;
                if (pk.active) {
                    float *q = j < pk.main_cols ? pk.base + (j >> 5) * pk.table_stride + int64_t(pk.rank[r]) * 32 + (j & 31)
                                                : pk.tail + int64_t(pk.rank[r]) * pk.tail_ld + (j - pk.main_cols);
                    *q = g * gnn_row_factor(pk.scale_mode, pk.counts[r]);
                } else if (G) {
                    G[r * ldg + j] = g;
                }
                s += g;
            }
        }
        red[threadIdx.x] = s;
        __syncthreads();
        if (rl == 0 && j < F) {
            float t = 0.0f;
            for (int k = 0; k < row_lanes; ++k) t += red[(k << log2_cols) + jl];
            partial[int64_t(blockIdx.x) * F + j] = t;
        }
        __syncthreads();
    }
}

// db[j] = sum of the block partials, in block order, two levels (chunks of 256 blocks).
__global__ void __launch_bounds__(256) colsum_reduce_kernel(const float *__restrict__ partial, int64_t n_blocks, int F,
                                                            float *__restrict__ out, int chunk) {
    const int64_t b0 = int64_t(blockIdx.x) * chunk;
    const int64_t b1 = b0 + chunk < n_blocks ? b0 + chunk : n_blocks;
    for (int j = threadIdx.x; j < F; j += blockDim.x) {
        float s = 0.0f;
        for (int64_t b = b0; b < b1; ++b) s += partial[b * F + j];
        out[int64_t(blockIdx.x) * F + j] = s;
    }
}

// Wt[c, r] = W[r, c] for a weight matrix (small next to everything else in a layer).  The products with W^T
// take the transposed copy as a row-contiguous operand: staged with 16-byte loads and stores, where the
// k-contiguous form of the same operand costs four 4-byte LDS stores per quad (dZ at 256 -> 256 on 2.45 M
// vertices: 4.2 -> 3.x ms).
__global__ void __launch_bounds__(256) transpose_kernel(const float *__restrict__ W, float *__restrict__ Wt, int rows, int cols) {
    const int64_t total = int64_t(rows) * cols;
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t t = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; t < total; t += stride) {
        const int64_t c = t / rows, r = t - c * rows;  // consecutive threads write consecutive elements of Wt
        Wt[t] = W[r * cols + c];
    }
}

__global__ void __launch_bounds__(256) zero_kernel(float *__restrict__ p, int64_t n) {
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t t = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; t < n; t += stride) p[t] = 0.0f;
}

int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

bool aggregate_first(int order, int64_t Fi, int64_t Fo) { return order == 1 || (order == 0 && Fi <= Fo); }

// Row stride of the matrices that the transform-first order gathers from (X W, and the masked
// output gradient): whole 16-byte groups, so that 16-byte loads apply to widths like 47.
int64_t gather_ld(int64_t Fo) { return round_up(Fo, 4); }

struct BwdLayout {
    int64_t g_off, t_off, part_off, part2_off, wt_off, mm_off, total;
    int64_t total_unfolded;  // with room for G behind everything else (aggregate first, rectifier, GNN_LAYER_NO_GATE_FOLD)
};

BwdLayout bwd_layout(int64_t N, int64_t Fi, int64_t Fo, bool agg_first, bool relu) {
    BwdLayout L{};
    int64_t off = 0;
    L.g_off = off;
    if (!agg_first) off += round_up(N * gather_ld(Fo) * 4, 256);  // aggregating first, the products read dH and H: no G
    L.t_off = off;
    off += round_up(N * (agg_first ? Fi : gather_ld(Fo)) * 4, 256);
    const int64_t n_blocks = (N + kRowsPerBlock - 1) / kRowsPerBlock;
    L.part_off = off;
    off += round_up(n_blocks * Fo * 4, 256);
    L.part2_off = off;
    off += round_up(((n_blocks + 255) / 256) * Fo * 4, 256);
    L.wt_off = off;
    off += round_up(Fi * Fo * 4, 256);  // W transposed
    L.mm_off = off;
    off += round_up(gnn_matmul_workspace_bytes(Fi, Fo, N), 256);
    L.total = off;
    L.total_unfolded = off;
    if (agg_first && relu) {
        L.g_off = off;
        L.total_unfolded = off + round_up(N * Fo * 4, 256);
    }
    return L;
}

}  // namespace

extern "C" GNN_API int64_t gnn_sage_layer_saved_elems(int64_t N, int64_t F_in, int64_t F_out, int order) {
    if (N < 0 || F_in < 0 || F_out < 0) return 0;
    return N * (aggregate_first(order, F_in, F_out) ? F_in : gather_ld(F_out));
}

extern "C" GNN_API int64_t gnn_sage_layer_workspace_bytes(int64_t N, int64_t F_in, int64_t F_out, int relu, int order) {
    if (N <= 0 || F_in <= 0 || F_out <= 0) return 0;
    return bwd_layout(N, F_in, F_out, aggregate_first(order, F_in, F_out), relu != 0).total;
}

static int check_layer(const gnn_layer_opts *opts, int64_t N, int64_t Fi, int64_t Fo, gnn_layer_opts &o) {
    if (!opts) return GNN_ERR_INVALID_ARG;
    o = *opts;
    if (N < 0 || Fi < 0 || Fo < 0 || N > INT32_MAX || Fi > INT32_MAX || Fo > INT32_MAX) return GNN_ERR_INVALID_ARG;
    if (o.order < 0 || o.order > 2) return GNN_ERR_INVALID_ARG;
    if (!o.plan) return GNN_ERR_UNSUPPORTED;  // the aggregator needs the plan's degree counts
    if (o.plan->n_rows != N || o.plan->indptr_is_64 != (o.indptr_is_64 ? 1 : 0)) return GNN_ERR_INVALID_ARG;
    return GNN_OK;
}

extern "C" GNN_API int gnn_sage_layer_fwd(const void *indptr, const int32_t *indices, const float *X, const float *W,
                                          const float *bias, float *saved, float *H, int64_t N, int64_t F_in, int64_t F_out,
                                          const gnn_layer_opts *opts) {
    gnn_layer_opts o;
    int rc = check_layer(opts, N, F_in, F_out, o);
    if (rc != GNN_OK) return rc;
    if (N == 0 || F_out == 0) return GNN_OK;
    if (F_in == 0) return GNN_ERR_INVALID_ARG;
    if (!indptr || !X || !W || !saved || !H) return GNN_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(o.stream);
    gnn_opts a{};
    a.dtype = GNN_F32;
    a.indptr_is_64 = o.indptr_is_64;
    a.stream = o.stream;
    a.plan = o.plan;
    if (aggregate_first(o.order, F_in, F_out)) {
        rc = gnn_aggregate_fwd(indptr, indices, nullptr, X, saved, N, F_in, GNN_SAGE_GCN, &a);
        if (rc != GNN_OK) return rc;
        return gnn_matmul_impl(saved, F_in, 0, W, F_out, 0, H, F_out, N, F_out, F_in, bias, o.relu, nullptr, 0, stream);
    }
    const bool force = (o.flags & GNN_LAYER_FORCE_PRODUCER_LAYOUT) != 0;
    // X W goes straight into the tables the aggregation gathers from, when that call would copy it there anyway
    gnn_packed_target pk{};
    if (!(o.flags & GNN_LAYER_NO_PRODUCER_LAYOUT)) {
        rc = gnn_packed_target_for(o.plan, indptr, indices, N, F_out, GNN_SAGE_GCN, /*backward=*/false, force, stream, &pk);
        if (rc != GNN_OK) return rc;
    }
    if (pk.active) {
        rc = gnn_matmul_impl(X, F_in, 0, W, F_out, 0, nullptr, 0, N, F_out, F_in, nullptr, 0, nullptr, 0, stream, &pk);
        if (rc != GNN_OK) return rc;
        return gnn_aggregate_prepacked(indptr, indices, H, N, F_out, GNN_SAGE_GCN, &a, /*backward=*/false, force, bias, o.relu);
    }
    // else X W is written with padded rows (the padding is never written and never used: the gather
    // reads it with 16-byte loads and drops it)
    const int64_t ldp = gather_ld(F_out);
    rc = gnn_matmul_impl(X, F_in, 0, W, F_out, 0, saved, ldp, N, F_out, F_in, nullptr, 0, nullptr, 0, stream);
    if (rc != GNN_OK) return rc;
    a.ldx = ldp;
    a.flags = GNN_FLAG_PADDED_ROWS;
    return gnn_aggregate_fwd_epilogue(indptr, indices, saved, H, N, F_out, GNN_SAGE_GCN, &a, bias, o.relu);
}

extern "C" GNN_API int gnn_sage_layer_bwd(const void *indptr_t, const int32_t *indices_t, const float *X, const float *W,
                                          const float *saved, const float *H, const float *dH, float *dX, float *dW,
                                          float *db, int64_t N, int64_t F_in, int64_t F_out, const gnn_layer_opts *opts) {
    gnn_layer_opts o;
    int rc = check_layer(opts, N, F_in, F_out, o);
    if (rc != GNN_OK) return rc;
    if (F_in == 0 || F_out == 0) return GNN_OK;
    if (!W || !dH || !dW || (o.relu && !H)) return GNN_ERR_INVALID_ARG;
    const bool agg_first = aggregate_first(o.order, F_in, F_out);
    if (N > 0 && (!indptr_t || !X || (agg_first && !saved))) return GNN_ERR_INVALID_ARG;
    const BwdLayout L = bwd_layout(N > 0 ? N : 1, F_in, F_out, agg_first, o.relu != 0);
    const bool fold_gate = agg_first && !(o.flags & GNN_LAYER_NO_GATE_FOLD);
    if (N > 0 && (!o.workspace || o.workspace_bytes < (fold_gate ? L.total : L.total_unfolded) ||
                  reinterpret_cast<uintptr_t>(o.workspace) % 16))
        return GNN_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(o.stream);
    (void)hipGetLastError();
    char *ws = static_cast<char *>(o.workspace);
    if (N == 0) {
        zero_kernel<<<64, 256, 0, stream>>>(dW, F_in * F_out);
        if (db) zero_kernel<<<1, 256, 0, stream>>>(db, F_out);
        return hipGetLastError() == hipSuccess ? GNN_OK : GNN_ERR_LAUNCH;
    }
    const bool need_g = o.relu || !agg_first;  // transform first gathers G: always the padded copy
    const int64_t ldg = agg_first ? F_out : gather_ld(F_out);
    float *G = (need_g && !fold_gate) ? reinterpret_cast<float *>(ws + L.g_off) : nullptr;
    float *T = reinterpret_cast<float *>(ws + L.t_off);
    float *part = reinterpret_cast<float *>(ws + L.part_off);
    float *part2 = reinterpret_cast<float *>(ws + L.part2_off);
    void *mm_ws = ws + L.mm_off;
    const int64_t mm_bytes = L.total - L.mm_off;  // (the optional G lies behind L.total)

    // The matrix the backward aggregation gathers (G when transforming first, dZ = G W^T when aggregating
    // first) is written straight into that call's tables when it would copy it there anyway.
    const bool force = (o.flags & GNN_LAYER_FORCE_PRODUCER_LAYOUT) != 0;
    gnn_packed_target pk{};
    if (dX || !agg_first) {
        if (!(o.flags & GNN_LAYER_NO_PRODUCER_LAYOUT)) {
            rc = gnn_packed_target_for(o.plan, indptr_t, indices_t, N, agg_first ? F_in : F_out, GNN_SAGE_GCN, /*backward=*/true,
                                       force, stream, &pk);
            if (rc != GNN_OK) return rc;
        }
    }
    const gnn_packed_target pk_mask = agg_first ? gnn_packed_target{} : pk;

    // Aggregating first, G is an operand of the two products only: they read dH and H themselves and
    // apply the rectifier while staging the operand, and the weight-gradient product adds up the bias
    // gradient from the tiles it stages anyway; G is never written.

    // rectifier mask and bias gradient
    const int64_t n_blocks = (N + kRowsPerBlock - 1) / kRowsPerBlock;
    if (!fold_gate && (need_g || db)) {
        int log2_cols = 0;
        while ((1 << log2_cols) < F_out && log2_cols < 8) ++log2_cols;
        mask_colsum_kernel<<<static_cast<unsigned>(n_blocks), 256, 0, stream>>>(H, dH, G, ldg, part, N, int(F_out),
                                                                                o.relu ? 1 : 0, log2_cols, pk_mask);
        if (db) {
            const int64_t n2 = (n_blocks + 255) / 256;
            colsum_reduce_kernel<<<static_cast<unsigned>(n2), 256, 0, stream>>>(part, n_blocks, int(F_out), part2, 256);
            colsum_reduce_kernel<<<1, 256, 0, stream>>>(part2, n2, int(F_out), db, int(n2));
        }
        if (hipGetLastError() != hipSuccess) return GNN_ERR_LAUNCH;
    }
    const float *Gm = (need_g && !fold_gate) ? G : dH;
    const float *gate = (fold_gate && o.relu) ? H : nullptr;
    // dW = Z^T G on `st`, and with the gate folded also db = the column sums of G, added in plane order
    auto weight_gradient = [&](hipStream_t st) -> int {
        if (!fold_gate) return gnn_matmul_impl(saved, F_in, 1, Gm, F_out, 0, dW, F_out, F_in, F_out, N, nullptr, 0, mm_ws, mm_bytes, st);
        gnn_gemm_fold fold{};
        fold.b_gate = gate;
        fold.colsum = db ? part : nullptr;
        fold.colsum_planes = n_blocks;
        int rcw = gnn_matmul_impl(saved, F_in, 1, dH, F_out, 0, dW, F_out, F_in, F_out, N, nullptr, 0, mm_ws, mm_bytes, st, nullptr, &fold);
        if (rcw != GNN_OK || !db) return rcw;
        const int64_t n2 = (fold.n_planes + 255) / 256;
        colsum_reduce_kernel<<<static_cast<unsigned>(n2), 256, 0, st>>>(part, fold.n_planes, int(F_out), part2, 256);
        colsum_reduce_kernel<<<1, 256, 0, st>>>(part2, n2, int(F_out), db, int(n2));
        return hipGetLastError() == hipSuccess ? GNN_OK : GNN_ERR_LAUNCH;
    };

    gnn_opts a{};
    a.dtype = GNN_F32;
    a.indptr_is_64 = o.indptr_is_64;
    a.stream = o.stream;
    a.plan = o.plan;
    if (agg_first) {
        if (!dX) return weight_gradient(stream);
        // dZ = G W^T first; then fork: dW = Z^T G (matrix cores) on the side stream while the caller's
        // stream runs the gather-bound backward aggregation
        gnn_gemm_fold fold_a{};
        fold_a.a_gate = gate;
        float *Wt = reinterpret_cast<float *>(ws + L.wt_off);
        transpose_kernel<<<64, 256, 0, stream>>>(W, Wt, int(F_in), int(F_out));
        if (hipGetLastError() != hipSuccess) return GNN_ERR_LAUNCH;
        rc = gnn_matmul_impl(Gm, F_out, 0, Wt, F_in, 0, T, F_in, N, F_in, F_out, nullptr, 0, nullptr, 0, stream, &pk, &fold_a);
        if (rc != GNN_OK) return rc;
        hipStream_t side = side_stream();
        hipEvent_t fork = nullptr, join = nullptr;
        if (side && (hipEventCreateWithFlags(&fork, hipEventDisableTiming) != hipSuccess ||
                     hipEventCreateWithFlags(&join, hipEventDisableTiming) != hipSuccess)) {
            if (fork) (void)hipEventDestroy(fork);
            fork = join = nullptr;
            side = nullptr;
            (void)hipGetLastError();
        }
        if (side && (hipEventRecord(fork, stream) != hipSuccess || hipStreamWaitEvent(side, fork, 0) != hipSuccess)) {
            (void)hipEventDestroy(fork);
            (void)hipEventDestroy(join);
            return GNN_ERR_LAUNCH;
        }
        rc = weight_gradient(side ? side : stream);
        int rc2 = pk.active ? gnn_aggregate_prepacked(indptr_t, indices_t, dX, N, F_in, GNN_SAGE_GCN, &a, /*backward=*/true, force, nullptr, 0)
                            : gnn_aggregate_bwd(indptr_t, indices_t, nullptr, T, dX, N, F_in, GNN_SAGE_GCN, &a);
        if (side) {  // join, whatever happened above: the caller's stream must not run ahead of the side stream
            if (hipEventRecord(join, side) != hipSuccess || hipStreamWaitEvent(stream, join, 0) != hipSuccess) rc = GNN_ERR_LAUNCH;
            (void)hipEventDestroy(fork);  // released by the runtime once the recorded work has completed
            (void)hipEventDestroy(join);
        }
        return rc != GNN_OK ? rc : rc2;
    }
    a.ldy = ldg;
    if (pk.active) {
        rc = gnn_aggregate_prepacked(indptr_t, indices_t, T, N, F_out, GNN_SAGE_GCN, &a, /*backward=*/true, force, nullptr, 0);
    } else {
        a.ldx = ldg;
        a.flags = GNN_FLAG_PADDED_ROWS;
        rc = gnn_aggregate_bwd(indptr_t, indices_t, nullptr, Gm, T, N, F_out, GNN_SAGE_GCN, &a);
    }
    if (rc != GNN_OK) return rc;
    rc = gnn_matmul_impl(X, F_in, 1, T, ldg, 0, dW, F_out, F_in, F_out, N, nullptr, 0, mm_ws, mm_bytes, stream);
    if (rc != GNN_OK || !dX) return rc;
    float *Wt = reinterpret_cast<float *>(ws + L.wt_off);
    transpose_kernel<<<64, 256, 0, stream>>>(W, Wt, int(F_in), int(F_out));
    if (hipGetLastError() != hipSuccess) return GNN_ERR_LAUNCH;
    return gnn_matmul_impl(T, ldg, 0, Wt, F_in, 0, dX, F_in, N, F_in, F_out, nullptr, 0, nullptr, 0, stream);
}
