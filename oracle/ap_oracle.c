/*
 * CPU oracle for the general aggregation primitive.  TEST INFRASTRUCTURE ONLY.
 *
 * The primitive of Section 4.1 (Algorithm 1) with the whole operator table
 * (Table 1):
 *
 *     f_O[v, j] = (+) over the edges e = (u -> v) of row v of  f_V[u, j] (x) f_E[e, j]
 *
 * (x) in {add, sub, mul, div, copylhs, copyrhs}, (+) in {sum, max, min}.  Scalar
 * loops in CSR order; shares nothing with the HIP library and is never called
 * from the product path.
 *
 * Readings where the paper is silent:
 *   - The reduction starts from the identity of (+) (0, -inf, +inf) and a row
 *     without edges yields 0.  (Algorithm 1 starts every row at zero; taken
 *     literally a max-reduction would then never go below zero.)
 *   - f_E may have one column instead of d; the scalar then serves every
 *     feature column.
 *   - An optional edge-id array maps CSR position e to the row of f_E it uses
 *     (a transposed graph keeps addressing the edge features of the original).
 *   - max / min also report WHICH edge won: the lowest CSR position among the
 *     edges that attain the extremum; -1 for an empty row.
 *   - sum: messages and sums in fp64.  max / min: the message is ONE fp32
 *     operation on fp32 inputs (correctly rounded, no contraction), because
 *     the comparison that picks the winner must see the values the fp32 kernel
 *     sees; the result is then exact, not approximate.
 *   - Backward (not in the paper): the derivative of the above.  For max /
 *     min only the winning edge of each (v, j) carries gradient.
 *
 * Pins (tests/test_oracle_ap_pins.py): an independent numpy formulation on
 * small graphs (per-edge message table, then ufunc.at reductions), the
 * copylhs/sum case against the dense adjacency product, closed forms, central
 * finite differences of an fp64 numpy forward for both gradients, and the
 * adjoint identity for the sum reducer.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

enum { BIN_ADD = 0, BIN_SUB = 1, BIN_MUL = 2, BIN_DIV = 3, BIN_COPY_LHS = 4, BIN_COPY_RHS = 5 };
enum { RED_SUM = 0, RED_MAX = 1, RED_MIN = 2 };

static double message64(int bin, double x, double y) {
    switch (bin) {
        case BIN_ADD: return x + y;
        case BIN_SUB: return x - y;
        case BIN_MUL: return x * y;
        case BIN_DIV: return x / y;
        case BIN_COPY_LHS: return x;
        default: return y;
    }
}

static float message32(int bin, float x, float y) {
    volatile float r;  /* one rounding to fp32, whatever the compiler would like to fuse */
    switch (bin) {
        case BIN_ADD: r = x + y; break;
        case BIN_SUB: r = x - y; break;
        case BIN_MUL: r = x * y; break;
        case BIN_DIV: r = x / y; break;
        case BIN_COPY_LHS: r = x; break;
        default: r = y; break;
    }
    return r;
}

/*
 * Forward.  indptr int64[N+1], indices int32[E]; eid int64[E] or NULL; fV
 * [*, ldv] fp32 (unused for copyrhs), fE [*, lde] fp32 with `ewidth` columns in
 * use (d or 1; unused for copylhs).  O [N, d] fp64; S [N, d] fp64 or NULL
 * receives the sum of |message| (sum reducer only); arg int64[N, d] or NULL
 * receives the winning CSR position (max / min only).
 */
int oracle_ap_fwd(const int64_t *indptr, const int32_t *indices, const int64_t *eid,
                  const float *fV, int64_t ldv, const float *fE, int64_t lde, int64_t ewidth,
                  double *O, double *S, int64_t *arg, int64_t N, int64_t d, int bin, int red) {
    if (bin < 0 || bin > 5 || red < 0 || red > 2) return 1;
    if (ewidth != d && ewidth != 1) return 2;
    if (bin != BIN_COPY_RHS && !fV) return 3;
    if (bin != BIN_COPY_LHS && !fE) return 4;
    /* rows are independent, so threads over rows change nothing in the results */
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t v = 0; v < N; ++v) {
        for (int64_t j = 0; j < d; ++j) {
            double acc = 0.0, mag = 0.0;
            float best = 0.0f;
            int64_t won = -1;
            for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e) {
                int64_t u = indices[e];
                int64_t r = eid ? eid[e] : e;
                float x = bin != BIN_COPY_RHS ? fV[u * ldv + j] : 0.0f;
                float y = bin != BIN_COPY_LHS ? fE[r * lde + (ewidth == 1 ? 0 : j)] : 0.0f;
                if (red == RED_SUM) {
                    double m = message64(bin, (double)x, (double)y);
                    acc += m;
                    mag += fabs(m);
                } else {
                    float m = message32(bin, x, y);
                    if (won < 0 || (red == RED_MAX ? m > best : m < best)) {
                        best = m;
                        won = e;
                    }
                }
            }
            if (red == RED_SUM) {
                O[v * d + j] = acc;
                if (S) S[v * d + j] = mag;
            } else {
                O[v * d + j] = won >= 0 ? (double)best : 0.0;
                if (arg) arg[v * d + j] = won;
            }
        }
    }
    return 0;
}

/*
 * Backward: gradients of sum_{v,j} dO[v,j] * f_O[v,j] with respect to f_V and
 * f_E.  With m = x (x) y:
 *     add: dm/dx = 1, dm/dy = 1       sub: 1, -1        mul: y, x
 *     div: 1/y, -x/y^2                copylhs: 1, 0     copyrhs: 0, 1
 * sum reducer: every edge contributes; max / min: only the edge arg[v, j].
 * dV [NV, d] fp64 (NV = rows of f_V), dE [NE, ewidth] fp64; with ewidth == 1
 * the edge gradient is summed over the feature columns.  SV / SE (optional)
 * receive the sums of the absolute terms.  All outputs are zero-filled here.
 */
int oracle_ap_bwd(const int64_t *indptr, const int32_t *indices, const int64_t *eid,
                  const float *fV, int64_t ldv, const float *fE, int64_t lde, int64_t ewidth,
                  const float *dO, int64_t ldo, const int64_t *arg,
                  double *dV, double *SV, int64_t NV, double *dE, double *SE, int64_t NE,
                  int64_t N, int64_t d, int bin, int red) {
    if (bin < 0 || bin > 5 || red < 0 || red > 2) return 1;
    if (ewidth != d && ewidth != 1) return 2;
    if (red != RED_SUM && !arg) return 5;
    if (dV) for (int64_t i = 0; i < NV * d; ++i) dV[i] = 0.0;
    if (SV) for (int64_t i = 0; i < NV * d; ++i) SV[i] = 0.0;
    if (dE) for (int64_t i = 0; i < NE * ewidth; ++i) dE[i] = 0.0;
    if (SE) for (int64_t i = 0; i < NE * ewidth; ++i) SE[i] = 0.0;
    for (int64_t v = 0; v < N; ++v) {
        for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e) {
            int64_t u = indices[e];
            int64_t r = eid ? eid[e] : e;
            for (int64_t j = 0; j < d; ++j) {
                if (red != RED_SUM && arg[v * d + j] != e) continue;
                double x = (bin != BIN_COPY_RHS && fV) ? (double)fV[u * ldv + j] : 0.0;
                double y = (bin != BIN_COPY_LHS && fE) ? (double)fE[r * lde + (ewidth == 1 ? 0 : j)] : 0.0;
                double g = (double)dO[v * ldo + j];
                double gx, gy;
                switch (bin) {
                    case BIN_ADD: gx = g; gy = g; break;
                    case BIN_SUB: gx = g; gy = -g; break;
                    case BIN_MUL: gx = g * y; gy = g * x; break;
                    case BIN_DIV: gx = g / y; gy = -g * x / (y * y); break;
                    case BIN_COPY_LHS: gx = g; gy = 0.0; break;
                    default: gx = 0.0; gy = g; break;
                }
                if (dV) {
                    dV[u * d + j] += gx;
                    if (SV) SV[u * d + j] += fabs(gx);
                }
                if (dE) {
                    int64_t k = r * ewidth + (ewidth == 1 ? 0 : j);
                    dE[k] += gy;
                    if (SE) SE[k] += fabs(gy);
                }
            }
        }
    }
    return 0;
}
