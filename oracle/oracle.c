/*
 * CPU oracle for the neighbour-aggregation primitive.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the plain definition written out: scalar loops, fp64
 * accumulation, ascending edge order.  It shares no code, header, table or
 * helper with the HIP library and must never be called from the product path;
 * only the tests, the smoke check and the bench's cpu_baseline leg use it.
 *
 * What is defined where in the paper:
 *   - Aggregation primitive, pull model over a destination-indexed CSR whose
 *     row v lists the sources u of edges u->v; the output row is zero before
 *     the neighbour loop; one owner per output row (Section 4.1, Algorithm 1).
 *   - The operators used here are rows of Table 1: (x) = copylhs (no edge
 *     data) or mul by a scalar edge feature, (+) = sum.
 *   - The primitive equals the sparse-times-dense product f_O = A x f_X
 *     (Section 2.1).
 *   - The paper does not spell out the backward pass, the mean divisor, the
 *     symmetric normalisation or empty rows; the readings taken are stated at
 *     each function below.
 *
 * Pins (tests/test_oracle_pins.py): dense adjacency product on graphs of at
 * most 64 vertices, all-ones-feature invariant, adjoint identity, closed forms
 * (rings, star, regular graph), relabelling equivariance, linearity, and brute
 * force recounts for the transpose and the degree-binning plan.  No function
 * in this file is "parity unpinned"; what IS unpinned is the numerical value
 * of Y on the large synthetic workloads, for which no printed example exists.
 *
 * The only parallelism is an OpenMP loop over output rows with dynamic
 * scheduling in chunks of contiguous rows (the scheduling Section 4.2
 * "Multithreading" describes); rows are independent, so results do not depend
 * on the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { OP_SUM = 0, OP_MEAN = 1, OP_GCN_SYM = 2, OP_SAGE_GCN = 3 };

static int64_t at_least_one(int64_t d) { return d > 0 ? d : 1; }

int oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Forward aggregation (Algorithm 1 with (+) = sum).
 *
 *   Y[v, :] = sum over e in row v of c_e * X[indices[e], :]
 *
 * c_e = 1 (copylhs), times w[e] if explicit edge weights are given (mul).
 * MEAN: the row sum is divided by the row length din[v] (number of stored
 *       edges, duplicates counted); an empty row stays zero.
 * GCN_SYM without explicit weights: c_e = 1/sqrt(max(dout[u],1)*max(din[v],1))
 *       with dout[u] the number of edges leaving u.  With explicit weights the
 *       weights are used as given (they already carry the normalisation).
 * SAGE_GCN: the aggregator of the paper's own runs (Section 6.1): the row sum,
 *       plus the vertex's own feature vector, divided by din[v] + 1 (the number
 *       of vectors added up; the paper says "normalizes with respect to the
 *       in-degree", and its Table 8 counts 51.5 = 50.5 + 1 vectors per vertex).
 *
 * rows == NULL: compute all N rows, Y is [N, F].  Otherwise compute only
 * rows[0..nrows), Y is [nrows, F] in that order (rows are independent in the
 * definition, so this is the same arithmetic).
 * S (optional, same shape as Y) receives sum_e |c_e * X[u_e, j]| (after the
 * MEAN division), the scale a rounding-error bound is stated against.
 */
int oracle_aggregate_fwd(const int64_t *indptr, const int32_t *indices, const float *w,
                         const float *X, int64_t ldx, double *Y, double *S,
                         int64_t N, int64_t F, int op, const int64_t *dout,
                         const int64_t *rows, int64_t nrows, int nthreads) {
    if (op < 0 || op > 3) return 1;
    if (op == OP_GCN_SYM && !w && !dout) return 2;
    int64_t count = rows ? nrows : N;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 64) num_threads(nthreads)
    for (int64_t i = 0; i < count; ++i) {
        int64_t v = rows ? rows[i] : i;
        double *acc = Y + i * F;
        double *mag = S ? S + i * F : NULL;
        for (int64_t j = 0; j < F; ++j) acc[j] = 0.0;
        if (mag) for (int64_t j = 0; j < F; ++j) mag[j] = 0.0;
        int64_t din = indptr[v + 1] - indptr[v];
        for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e) {
            int64_t u = indices[e];
            double c = 1.0;
            if (w) c = (double)w[e];
            else if (op == OP_GCN_SYM)
                c = 1.0 / sqrt((double)at_least_one(dout[u]) * (double)at_least_one(din));
            const float *x = X + u * ldx;
            for (int64_t j = 0; j < F; ++j) {
                double t = c * (double)x[j];
                acc[j] += t;
                if (mag) mag[j] += fabs(t);
            }
        }
        if (op == OP_MEAN && din > 0) {
            for (int64_t j = 0; j < F; ++j) acc[j] /= (double)din;
            if (mag) for (int64_t j = 0; j < F; ++j) mag[j] /= (double)din;
        }
        if (op == OP_SAGE_GCN) {
            const float *self = X + v * ldx;
            for (int64_t j = 0; j < F; ++j) {
                acc[j] = (acc[j] + (double)self[j]) / (double)(din + 1);
                if (mag) mag[j] = (mag[j] + fabs((double)self[j])) / (double)(din + 1);
            }
        }
    }
    return 0;
}

/*
 * Backward aggregation: the exact adjoint of the forward linear map, taken
 * over the transposed graph (row u of the transposed CSR lists the
 * destinations v of edges u->v; wt is w in that edge order).
 *
 *   dX[u, :] = sum over e' in transposed row u of c_e' * dY[indices_t[e'], :]
 *
 * SUM: c = wt or 1.  MEAN: additionally divided by din[v] of the GATHERED
 * vertex v (the forward pass divided output row v by din[v]).  GCN_SYM without
 * weights: the same 1/sqrt(max(dout[u],1)*max(din[v],1)) as forward, where
 * dout[u] is this row's length.  SAGE_GCN: every edge term is divided by
 * din[v] + 1 of the gathered vertex, and the row's own gradient enters as
 * dY[u] / (din[u] + 1) (the transpose of adding the self vector).  din is the
 * forward in-degree vector, needed for MEAN, SAGE_GCN and weight-less GCN_SYM.
 */
int oracle_aggregate_bwd(const int64_t *indptr_t, const int32_t *indices_t, const float *wt,
                         const float *dY, int64_t ldy, double *dX, double *S,
                         int64_t N, int64_t F, int op, const int64_t *din,
                         const int64_t *rows, int64_t nrows, int nthreads) {
    if (op < 0 || op > 3) return 1;
    if ((op == OP_MEAN || op == OP_SAGE_GCN) && !din) return 2;
    if (op == OP_GCN_SYM && !wt && !din) return 2;
    int64_t count = rows ? nrows : N;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 64) num_threads(nthreads)
    for (int64_t i = 0; i < count; ++i) {
        int64_t u = rows ? rows[i] : i;
        double *acc = dX + i * F;
        double *mag = S ? S + i * F : NULL;
        for (int64_t j = 0; j < F; ++j) acc[j] = 0.0;
        if (mag) for (int64_t j = 0; j < F; ++j) mag[j] = 0.0;
        int64_t dout = indptr_t[u + 1] - indptr_t[u];
        for (int64_t e = indptr_t[u]; e < indptr_t[u + 1]; ++e) {
            int64_t v = indices_t[e];
            double c = 1.0;
            if (wt) c = (double)wt[e];
            else if (op == OP_GCN_SYM)
                c = 1.0 / sqrt((double)at_least_one(dout) * (double)at_least_one(din[v]));
            if (op == OP_MEAN) c /= (double)din[v]; /* v has at least this edge, so din[v] >= 1 */
            if (op == OP_SAGE_GCN) c /= (double)(din[v] + 1);
            const float *g = dY + v * ldy;
            for (int64_t j = 0; j < F; ++j) {
                double t = c * (double)g[j];
                acc[j] += t;
                if (mag) mag[j] += fabs(t);
            }
        }
        if (op == OP_SAGE_GCN) {
            const float *self = dY + u * ldy;
            for (int64_t j = 0; j < F; ++j) {
                double t = (double)self[j] / (double)(din[u] + 1);
                acc[j] += t;
                if (mag) mag[j] += fabs(t);
            }
        }
    }
    return 0;
}

/*
 * Row pointers of the destination-indexed CSR from a destination array that
 * is already sorted ascending: indptr[v] = number of edges with dst < v.
 */
int oracle_csr_indptr(const int32_t *dst_sorted, int64_t E, int64_t N, int64_t *indptr) {
    for (int64_t v = 0; v <= N; ++v) indptr[v] = 0;
    for (int64_t e = 0; e < E; ++e) {
        int64_t v = dst_sorted[e];
        if (v < 0 || v >= N) return 1;
        if (e > 0 && dst_sorted[e - 1] > dst_sorted[e]) return 2;
        indptr[v + 1] += 1;
    }
    for (int64_t v = 0; v < N; ++v) indptr[v + 1] += indptr[v];
    return 0;
}

/*
 * Transposed graph by a stable counting sort on the source id: edges of
 * transposed row u keep their relative order from the CSR (so, for a CSR with
 * ascending neighbours, ascending destination).  perm[e'] is the CSR position
 * of transposed edge e', i.e. indices_t[e'] = dst(perm[e']) and, for weights,
 * wt[e'] = w[perm[e']].
 */
int oracle_transpose(const int64_t *indptr, const int32_t *indices, int64_t N,
                     int64_t *indptr_t, int32_t *indices_t, int64_t *perm) {
    int64_t E = indptr[N];
    for (int64_t u = 0; u <= N; ++u) indptr_t[u] = 0;
    for (int64_t e = 0; e < E; ++e) {
        int64_t u = indices[e];
        if (u < 0 || u >= N) return 1;
        indptr_t[u + 1] += 1;
    }
    for (int64_t u = 0; u < N; ++u) indptr_t[u + 1] += indptr_t[u];
    int64_t *cursor = (int64_t *)malloc(sizeof(int64_t) * (size_t)(N > 0 ? N : 1));
    if (!cursor) return 3;
    memcpy(cursor, indptr_t, sizeof(int64_t) * (size_t)N);
    for (int64_t v = 0; v < N; ++v) {
        for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e) {
            int64_t u = indices[e];
            int64_t pos = cursor[u]++;
            indices_t[pos] = (int32_t)v;
            perm[pos] = e;
        }
    }
    free(cursor);
    return 0;
}

/*
 * Degree-binning plan (the GPU-side replacement for dynamic scheduling over
 * rows of very different length, Section 4.2 "Multithreading").
 *
 * thresholds t[0] < t[1] < ... < t[k-1] (all > 0) cut the degree axis into
 * k+1 bins: bin(v) = number of thresholds <= deg(v).  row_perm lists the rows
 * bin after bin, ascending row id inside a bin; bin_offsets[b] is where bin b
 * starts in row_perm (k+2 entries).  If hub_chunk > 0 every row of the LAST
 * bin is cut into consecutive pieces of hub_chunk edges (the last piece may be
 * shorter); pieces are listed in row_perm order, then ascending position, as
 * triples (row, e_begin, e_end).  Returns the number of pieces through
 * *n_chunks; if chunks == NULL only counts them.
 */
int oracle_plan(const int64_t *indptr, int64_t N, const int64_t *thresholds, int k,
                int64_t hub_chunk, int64_t *bin_offsets, int32_t *row_perm,
                int64_t *chunks, int64_t *n_chunks) {
    int nb = k + 1;
    for (int b = 0; b <= nb; ++b) bin_offsets[b] = 0;
    for (int64_t v = 0; v < N; ++v) {
        int64_t d = indptr[v + 1] - indptr[v];
        int b = 0;
        for (int i = 0; i < k; ++i) if (thresholds[i] <= d) b += 1;
        bin_offsets[b + 1] += 1;
    }
    for (int b = 0; b < nb; ++b) bin_offsets[b + 1] += bin_offsets[b];
    int64_t *cursor = (int64_t *)malloc(sizeof(int64_t) * (size_t)nb);
    if (!cursor) return 3;
    for (int b = 0; b < nb; ++b) cursor[b] = bin_offsets[b];
    for (int64_t v = 0; v < N; ++v) {
        int64_t d = indptr[v + 1] - indptr[v];
        int b = 0;
        for (int i = 0; i < k; ++i) if (thresholds[i] <= d) b += 1;
        row_perm[cursor[b]++] = (int32_t)v;
    }
    free(cursor);
    int64_t nc = 0;
    if (hub_chunk > 0) {
        for (int64_t p = bin_offsets[nb - 1]; p < bin_offsets[nb]; ++p) {
            int64_t v = row_perm[p];
            for (int64_t b = indptr[v]; b < indptr[v + 1]; b += hub_chunk) {
                int64_t e = b + hub_chunk < indptr[v + 1] ? b + hub_chunk : indptr[v + 1];
                if (chunks) {
                    chunks[3 * nc + 0] = v;
                    chunks[3 * nc + 1] = b;
                    chunks[3 * nc + 2] = e;
                }
                nc += 1;
            }
        }
    }
    *n_chunks = nc;
    return 0;
}
